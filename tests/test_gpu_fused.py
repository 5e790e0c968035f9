"""GPU parity of the depth-fused forward pass: every layer of every scheduled job
in one launch, workgroups of layer l+1 waiting on the device for the job's layer
l.  It computes each tile exactly like the per-depth launches, so its outputs
must be bit-identical to theirs and within tolerance of the oracle."""
import numpy as np
import pytest
import torch

from oracle import dense
from paper_1902_04610_amd import salus, synth
from gpu_util import DevicePool, mlp_layout, norm_rel_err
from test_gpu_kernels import run_jobs, TOL_BF16_TIGHT, TOL_F32

pytestmark = pytest.mark.gpu

GELU, RELU, NONE = salus.ACT_GELU, salus.ACT_RELU, salus.ACT_NONE


def both_ways(jobs, dtype):
    fused, refs, fused_launches = run_jobs(jobs, dtype, fuse=True)
    plain, _, plain_launches = run_jobs(jobs, dtype, fuse=False)
    for f, p, j in zip(fused, plain, jobs):
        assert np.array_equal(f.view(np.uint32), p.view(np.uint32)), j
    return fused, refs, fused_launches, plain_launches


def test_bf16_all_depths_in_one_launch():
    jobs = [dict(M=m, dims=(256, 1024, 256, 264), acts=[GELU, GELU, NONE]) for m in (1, 7, 16, 23, 32)]
    jobs += [dict(M=9, dims=(128, 136), acts=[RELU]),
             dict(M=32, dims=(64, 64, 64, 64, 64), acts=[RELU] * 3 + [NONE]),
             dict(M=5, dims=(512, 384, 128, 640, 256, 128, 72), acts=[GELU] * 5 + [NONE], strip=True)]
    outs, refs, fused_launches, plain_launches = both_ways(jobs, salus.BF16)
    assert fused_launches == 1 and plain_launches == 6
    for o, r, j in zip(outs, refs, jobs):
        assert np.isfinite(o).all(), j
        assert norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))


@pytest.mark.parametrize("M", [1, 16, 17, 32])
def test_bf16_packing_shapes_with_strip_weights(M):
    jobs = [dict(M=M, dims=(1024, 4096, 1024, 1024), acts=[GELU, GELU, NONE], strip=True) for _ in range(6)]
    outs, refs, fused_launches, _ = both_ways(jobs, salus.BF16)
    assert fused_launches == 1
    for o, r in zip(outs, refs):
        assert norm_rel_err(o, r) < TOL_BF16_TIGHT


@pytest.mark.parametrize("M", [1, 8, 19, 40, 67])
def test_f32_all_depths_in_one_launch(M):
    jobs = [dict(M=M, dims=d, acts=a) for d, a in
            [((256, 256, 256), [RELU, NONE]), ((64, 100, 36, 8), [GELU, RELU, NONE]), ((40, 12), [NONE])]]
    outs, refs, fused_launches, plain_launches = both_ways(jobs, salus.F32)
    assert fused_launches == 1 and plain_launches == 3
    for o, r, j in zip(outs, refs, jobs):
        assert norm_rel_err(o, r) < TOL_F32, (j, norm_rel_err(o, r))


def test_more_jobs_than_one_fused_launch_holds():
    jobs = [dict(M=1 + (i % 5), dims=(64, 72, 40), acts=[RELU, NONE]) for i in range(70)]
    outs, refs, fused_launches, _ = both_ways(jobs, salus.BF16)
    assert fused_launches == 2                  # 64 job slots per launch
    for o, r in zip(outs, refs):
        assert norm_rel_err(o, r) < TOL_BF16_TIGHT


def test_jobs_the_fused_launch_does_not_take_fall_back_to_one_launch_per_depth():
    # 40 rows (bf16) is above what the weight-streaming kernels are used for;
    # seven layers are more than one fused launch holds
    for jobs, launches in [([dict(M=40, dims=(64, 72, 40), acts=[RELU, NONE]),
                             dict(M=4, dims=(64, 72, 40), acts=[RELU, NONE])], 4),   # per depth: up to 32 rows, above
                           ([dict(M=3, dims=(64,) * 8, acts=[RELU] * 6 + [NONE])], 7)]:
        outs, refs, fused_launches, plain_launches = both_ways(jobs, salus.BF16)
        assert fused_launches == plain_launches == launches
        for o, r in zip(outs, refs):
            assert norm_rel_err(o, r) < TOL_BF16_TIGHT


class Fleet:
    """A pool with resident bf16 models whose rounds name changing subsets and
    row counts: what the descriptor cache and the alternating counters see."""

    def __init__(self, n_jobs, dims, acts, max_m, seed, fuse=True):
        self.dims, self.acts, self.max_m = dims, acts, max_m
        self.w_offs, P, self.x_off, self.y_off, self.h_off, E = mlp_layout(dims, 2, max_m)
        cap = (n_jobs * (P + E) + 4096 + 255) // 256 * 256
        self.dp = DevicePool(cap, policy=salus.POLICY_PACK, fuse_depths=fuse)
        rng = np.random.default_rng(seed)
        self.jobs, self.W = [], []
        for _ in range(n_jobs):
            st, jid = self.dp.pool.lane_alloc(P, E, 0, 0)
            assert st == salus.OK
            q = self.dp.pool.job_query(jid)
            Ws = [synth.f32_to_bf16_bits((rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32))
                  for K, N in zip(dims[:-1], dims[1:])]
            for w, off in zip(Ws, self.w_offs):
                self.dp.write(q.persist_off + off, w)
            self.jobs.append(jid)
            self.W.append(Ws)
        self.rng = rng

    def round(self, active, rows):
        """Runs jobs `active` with `rows[i]` rows each; returns (gpu, oracle) outputs."""
        items, refs = [], []
        for idx, M in zip(active, rows):
            jid = self.jobs[idx]
            q = self.dp.pool.job_query(jid)
            X = synth.f32_to_bf16_bits(self.rng.uniform(-1, 1, (M, self.dims[0])).astype(np.float32))
            self.dp.write(q.lane_off + self.x_off, X)
            self.dp.write(q.lane_off + self.y_off, np.full((M, self.dims[-1]), np.nan, np.float32))
            items.append(dict(job=jid, M=M, dtype=salus.BF16, x_off=self.x_off, y_off=self.y_off,
                              h_off=self.h_off,
                              layers=[(K, N, off, a) for K, N, off, a in
                                      zip(self.dims[:-1], self.dims[1:], self.w_offs, self.acts)]))
            refs.append(dense.mlp_forward_bf16(X, self.W[idx], self.acts)[-1])
        descs, keep = salus.Pool.make_descs(items)
        assert self.dp.pool.grouped_forward(descs, stream=self.dp.stream) == salus.OK
        self.dp.sync()
        outs = []
        for idx, M in zip(active, rows):
            q = self.dp.pool.job_query(self.jobs[idx])
            outs.append(self.dp.read(q.lane_off + self.y_off, M * self.dims[-1] * 4, np.float32)
                        .reshape(M, self.dims[-1]).copy())
        return outs, refs


def test_rounds_with_changing_jobs_and_rows_reuse_cached_descriptors():
    fleet = Fleet(12, (128, 384, 136, 72), [GELU, RELU, NONE], 32, seed=11)
    rng = np.random.default_rng(12)
    for r in range(9):
        k = int(rng.integers(1, 13))
        active = sorted(rng.choice(12, size=k, replace=False).tolist())
        rows = [int(rng.integers(1, 33)) for _ in active]
        outs, refs = fleet.round(active, rows)
        assert fleet.dp.pool.fused_check() == salus.OK
        for o, ref, a, m in zip(outs, refs, active, rows):
            assert np.isfinite(o).all(), (r, a, m)
            assert norm_rel_err(o, ref) < TOL_BF16_TIGHT, (r, a, m)
    assert fleet.dp.pool.stats()["gemm_launches"] == 9
    fleet.dp.close()


def test_descriptors_follow_a_job_that_moves():
    # job 0 leaves: the younger lanes slide, every lane address changes; the cached
    # descriptors must not be used as they are
    fleet = Fleet(4, (64, 128, 72), [RELU, NONE], 8, seed=13)
    outs, refs = fleet.round([0, 1, 2, 3], [8, 3, 5, 1])
    for o, ref in zip(outs, refs):
        assert norm_rel_err(o, ref) < TOL_BF16_TIGHT
    before = fleet.dp.pool.job_query(fleet.jobs[2]).lane_off
    assert fleet.dp.pool.lane_free(fleet.jobs[0]) == salus.OK
    assert fleet.dp.pool.job_query(fleet.jobs[2]).lane_off != before
    outs, refs = fleet.round([1, 2, 3], [2, 8, 4])
    for o, ref in zip(outs, refs):
        assert norm_rel_err(o, ref) < TOL_BF16_TIGHT
    assert fleet.dp.pool.fused_check() == salus.OK
    fleet.dp.close()


def test_a_wait_that_gives_up_is_reported_and_the_pool_stays_usable():
    # With a budget of zero polls a consumer gives up unless its input is already
    # complete when it first looks.  All 64 workgroups of this round are resident
    # at once and the first layer streams 8 MB per job, so the second layer looks
    # long before.  Every workgroup still runs to its end.
    fleet = Fleet(4, (4096, 1024, 1024), [RELU, NONE], 16, seed=14)
    pool = fleet.dp.pool
    assert pool.fused_spin_limit(0) == salus.OK
    fleet.round([0, 1, 2, 3], [16, 16, 16, 16])
    assert pool.fused_check() == salus.ETIMEOUT
    assert "gave up" in pool.last_error()
    assert pool.fused_check() == salus.OK              # reported once
    assert pool.stats()["fused_timeouts"] == 1
    assert pool.fused_spin_limit(1 << 21) == salus.OK
    outs, refs = fleet.round([0, 1, 2, 3], [16, 9, 1, 16])
    assert pool.fused_check() == salus.OK
    for o, ref in zip(outs, refs):
        assert norm_rel_err(o, ref) < TOL_BF16_TIGHT
    fleet.dp.close()


def run_mixed_dtypes(fuse):
    """Float and bf16 jobs of different depths in ONE packed iteration."""
    specs = [(salus.F32, 6, (64, 100, 36)), (salus.BF16, 9, (128, 136, 72, 40)), (salus.F32, 20, (40, 12)),
             (salus.BF16, 32, (256, 264))]
    acts_of = lambda dims: [RELU] * (len(dims) - 2) + [NONE]
    layouts = [mlp_layout(d, 4 if dt == salus.F32 else 2, m) for dt, m, d in specs]
    cap = (sum(l[1] + l[5] for l in layouts) + 4096 + 255) // 256 * 256
    dp = DevicePool(cap, policy=salus.POLICY_PACK, fuse_depths=fuse)
    rng = np.random.default_rng(31)
    items, refs = [], []
    for (dt, M, dims), (w_offs, P, x_off, y_off, h_off, E) in zip(specs, layouts):
        st, jid = dp.pool.lane_alloc(P, E, 0, 0)
        assert st == salus.OK
        q = dp.pool.job_query(jid)
        Ws = [(rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32) for K, N in zip(dims[:-1], dims[1:])]
        X = rng.uniform(-1, 1, (M, dims[0])).astype(np.float32)
        if dt == salus.BF16:
            Ws, X = [synth.f32_to_bf16_bits(w) for w in Ws], synth.f32_to_bf16_bits(X)
        for w, off in zip(Ws, w_offs):
            dp.write(q.persist_off + off, w)
        dp.write(q.lane_off + x_off, X)
        dp.write(q.lane_off + y_off, np.full((M, dims[-1]), np.nan, np.float32))
        acts = acts_of(dims)
        items.append(dict(job=jid, M=M, dtype=dt, x_off=x_off, y_off=y_off, h_off=h_off,
                          layers=[(K, N, off, a) for K, N, off, a in zip(dims[:-1], dims[1:], w_offs, acts)]))
        fwd = dense.mlp_forward_f32 if dt == salus.F32 else dense.mlp_forward_bf16
        refs.append(fwd(X, Ws, acts)[-1])
    descs, keep = salus.Pool.make_descs(items)
    assert dp.pool.grouped_forward(descs, stream=dp.stream) == salus.OK
    dp.sync()
    assert dp.pool.fused_check() == salus.OK
    outs = []
    for it, (dt, M, dims) in zip(items, specs):
        q = dp.pool.job_query(it["job"])
        outs.append(dp.read(q.lane_off + it["y_off"], M * dims[-1] * 4, np.float32).reshape(M, dims[-1]).copy())
    launches = dp.pool.stats()["gemm_launches"]
    dp.close()
    return outs, refs, launches, [dt for dt, _, _ in specs]


def test_float_and_bf16_jobs_in_one_round_both_ways():
    fused, refs, fused_launches, dts = run_mixed_dtypes(True)
    plain, _, plain_launches, _ = run_mixed_dtypes(False)
    assert fused_launches == 2                 # one launch per dtype
    assert plain_launches == 2 + 3             # float jobs: 2 depths, bf16 jobs: 3
    for f, p, r, dt in zip(fused, plain, refs, dts):
        assert np.array_equal(f.view(np.uint32), p.view(np.uint32))
        assert norm_rel_err(f, r) < (TOL_F32 if dt == salus.F32 else TOL_BF16_TIGHT)
