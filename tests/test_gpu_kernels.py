"""GPU parity of the individual kernels, through the C ABI, against the oracle."""
import numpy as np
import pytest
import torch

from oracle import dense
from paper_1902_04610_amd import salus, synth
from gpu_util import DevicePool, mlp_layout, norm_rel_err

pytestmark = pytest.mark.gpu

# Tolerances (max |gpu - oracle| / max |oracle| per output matrix).
#  fp32: products and sums in float; K <= 4096 terms of magnitude <= max|y|/sqrt(K)
#        each rounded to 2^-24 relative: well under 1e-5.
#  bf16: products of two bf16 numbers are exact in float, sums in float; the only
#        other difference is an occasional 1-ulp (2^-8) flip when an activation is
#        rounded to bf16 for the next layer.  2e-2 is the stated bound; 2e-3 is what
#        the arithmetic allows and is tight enough to expose a dropped k-term.
TOL_F32 = 1e-5
TOL_BF16 = 2e-2
TOL_BF16_TIGHT = 2e-3


def splitmix(seed, idx):
    with np.errstate(over="ignore"):
        z = np.uint64(seed) + idx.astype(np.uint64) * np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


@pytest.mark.parametrize("nbytes", [16, 48, 4096, 65536, 65536 + 16, 5 * 65536 + 4080, 37 * 1024 * 1024 + 32])
def test_copy_disjoint(nbytes):
    src = torch.randint(0, 256, (nbytes + 512,), dtype=torch.uint8, device="cuda")
    dst = torch.full((nbytes + 512,), 7, dtype=torch.uint8, device="cuda")
    salus.copy(dst.data_ptr() + 256, src.data_ptr() + 256, nbytes)
    torch.cuda.synchronize()
    assert torch.equal(dst[256:256 + nbytes], src[256:256 + nbytes])
    assert (dst[:256] == 7).all() and (dst[256 + nbytes:] == 7).all()      # nothing outside


@pytest.mark.parametrize("shift,nbytes", [(16, 4096), (256, 3 * 1024 * 1024 + 4096), (65536, 20 * 65536 + 48),
                                           (1 << 20, 9 * (1 << 20) + 512), (100 * 65536, 100 * 65536),
                                           # the in-place kernel's chunks are 192 KiB: shifts around one and
                                           # several chunks, and ranges of several rounds of its resident grid
                                           (196608 + 16, 7 * 196608 + 32), (3 * 196608 - 16, 50 * 196608), (196608 - 16, 196608 + 16),
                                           (196608, 9 * 196608 + 4096), (131072, 9 * 131072 + 4096), (48 * 1024, 300 * (1 << 20) + 4080),
                                           (5 * (1 << 20) + 256, 200 * (1 << 20))])
def test_copy_overlapping_toward_lower_addresses(shift, nbytes):
    rng = np.random.default_rng(shift)
    host = rng.integers(0, 256, nbytes + shift + 512, dtype=np.uint8)
    dev = torch.from_numpy(host).cuda()
    salus.copy(dev.data_ptr() + 256, dev.data_ptr() + 256 + shift, nbytes)
    torch.cuda.synchronize()
    want = host.copy()
    want[256:256 + nbytes] = host[256 + shift:256 + shift + nbytes]          # memmove
    assert np.array_equal(dev.cpu().numpy(), want)


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 1000, 4096])
def test_wavefront_scan_is_bit_exact(n):
    rng = np.random.default_rng(n)
    vals = [int(v) for v in rng.integers(0, 1 << 40, n)]
    vals[0] = (1 << 62) + 12345                      # exercises the upper bits
    scratch = torch.empty((2 * n + 2) * 8, dtype=torch.uint8, device="cuda")
    got = salus.scan_u64(vals, scratch.data_ptr())
    want, run = [], 0
    for v in vals:
        want.append(run)
        run += v
    assert got == want + [run]


def test_pattern_fill_and_check():
    n = 3 * 1024 * 1024 + 8
    buf = torch.zeros(n + 8, dtype=torch.uint8, device="cuda")
    scratch = torch.zeros(8, dtype=torch.uint8, device="cuda")
    salus.fill_pattern(buf.data_ptr(), n, 99)
    words = buf[:n].cpu().numpy().view(np.uint64)
    idx = np.array([0, 1, 2, 12345, n // 8 - 1])
    assert np.array_equal(words[idx], splitmix(99, idx))
    assert (buf[n:] == 0).all()
    assert salus.check_pattern(buf.data_ptr(), n, 99, scratch.data_ptr()) == 0
    buf[4096] ^= 1
    buf[n - 1] ^= 0x80
    assert salus.check_pattern(buf.data_ptr(), n, 99, scratch.data_ptr()) == 2
    assert salus.check_pattern(buf.data_ptr(), n, 100, scratch.data_ptr()) == n // 8


def run_jobs(jobs, dtype, fuse=False):
    """jobs: list of dict(M, dims, acts).  Builds one pool with a lane per job,
    runs them as ONE packed iteration and returns (gpu outputs, oracle outputs,
    launches).  fuse: the pool runs all layer depths in one launch."""
    esz = 2 if dtype == salus.BF16 else 4
    layouts = [mlp_layout(j["dims"], esz, j["M"]) for j in jobs]
    cap = sum(l[1] + l[5] for l in layouts) + 4096
    cap = (cap + 255) // 256 * 256
    dp = DevicePool(cap, policy=salus.POLICY_PACK, fuse_depths=fuse)
    rng = np.random.default_rng(len(jobs) * 100 + jobs[0]["M"])
    items, refs = [], []
    for j, (w_offs, P, x_off, y_off, h_off, E) in zip(jobs, layouts):
        st, jid = dp.pool.lane_alloc(P, E, 0, 1)
        assert st == salus.OK
        q = dp.pool.job_query(jid)
        dims, M = j["dims"], j["M"]
        # optional: w_scale / w_mean shape the pre-activations (mean w_mean * E[x] per output)
        Ws = [(j.get("w_scale", 1.0) * rng.standard_normal((K, N)) / np.sqrt(K) + j.get("w_mean", 0.0) / K)
              .astype(np.float32) for K, N in zip(dims[:-1], dims[1:])]
        X = rng.uniform(j.get("x_lo", -1), j.get("x_hi", 1), (M, dims[0])).astype(np.float32)
        if dtype == salus.BF16:
            Ws = [synth.f32_to_bf16_bits(w) for w in Ws]
            X = synth.f32_to_bf16_bits(X)
        # "strip": layers whose width allows it are stored in 128-column strips
        lay = [salus.LAYOUT_STRIP128 if j.get("strip") and dtype == salus.BF16 and w.shape[1] % 128 == 0
               else salus.LAYOUT_ROWMAJOR for w in Ws]
        for w, off, l in zip(Ws, w_offs, lay):
            dp.write(q.persist_off + off, salus.pack_strip128(w) if l else w)
        dp.write(q.lane_off + x_off, X)
        items.append(dict(job=jid, M=M, dtype=dtype, x_off=x_off, y_off=y_off, h_off=h_off,
                          layers=[(K, N, off, a, l) for K, N, off, a, l in
                                  zip(dims[:-1], dims[1:], w_offs, j["acts"], lay)]))
        fwd = dense.mlp_forward_bf16 if dtype == salus.BF16 else dense.mlp_forward_f32
        refs.append(fwd(X, Ws, j["acts"])[-1])
    # poison the outputs so that an unwritten element shows
    for it, j in zip(items, jobs):
        q = dp.pool.job_query(it["job"])
        dp.write(q.lane_off + it["y_off"], np.full((j["M"], j["dims"][-1]), np.nan, np.float32))
    sched = dp.pool.schedule_iteration(cap=len(jobs) + 1)
    assert [s[0] for s in sched] == [it["job"] for it in items]
    descs, keep = salus.Pool.make_descs(items)
    assert dp.pool.grouped_forward(descs, stream=dp.stream) == salus.OK
    dp.sync()
    assert dp.pool.fused_check() == salus.OK
    outs = []
    for it, j in zip(items, jobs):
        q = dp.pool.job_query(it["job"])
        outs.append(dp.read(q.lane_off + it["y_off"], j["M"] * j["dims"][-1] * 4, np.float32)
                    .reshape(j["M"], j["dims"][-1]).copy())
    launches = dp.pool.stats()["gemm_launches"]
    dp.close()
    return outs, refs, launches


GELU, RELU, NONE = salus.ACT_GELU, salus.ACT_RELU, salus.ACT_NONE


@pytest.mark.parametrize("M", [1, 5, 16, 17, 32, 33, 48, 64, 65, 70, 96, 127, 128])
def test_bf16_single_layer_ragged_shapes(M):
    jobs = [dict(M=M, dims=(K, N), acts=[act]) for K, N, act in
            [(8, 8, NONE), (40, 72, RELU), (136, 136, GELU), (1024, 520, NONE), (264, 128, GELU),
             (32, 1000, NONE)]]
    outs, refs, launches = run_jobs(jobs, salus.BF16)
    assert launches == (1 if M < 128 else 2)      # from 128 rows the layer with K % 64 == 0 goes to the tiled kernel
    for o, r, j in zip(outs, refs, jobs):
        assert np.isfinite(o).all(), j
        assert norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))


@pytest.mark.parametrize("M", [33, 64, 65, 128])
def test_bf16_rows_33_to_128_take_64_row_tiles_of_either_width(M):
    """Few jobs: 64-column tiles (more workgroups); many jobs: 128-column tiles.  Both
    read the weights once per 64 rows; ragged K, N and strips included."""
    shapes = [(72, 8, NONE), (136, 200, RELU), (1000, 520, GELU), (2048, 1000, NONE), (264, 128, GELU)]
    few = [dict(M=M, dims=(K, N), acts=[act]) for K, N, act in shapes]
    few.append(dict(M=M, dims=(256, 512, 384, 136), acts=[GELU, RELU, NONE], strip=True))
    outs, refs, launches = run_jobs(few, salus.BF16)
    for o, r, j in zip(outs, refs, few):
        assert np.isfinite(o).all(), j
        assert norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))
    many = [dict(M=max(M - (i % 3), 33), dims=(40, 1000), acts=[[NONE, RELU, GELU][i % 3]]) for i in range(40)]
    outs, refs, launches = run_jobs(many, salus.BF16)           # 40 jobs x 8 column tiles >= 256
    assert launches == 1
    for o, r, j in zip(outs, refs, many):
        assert np.isfinite(o).all() and norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))


def test_bf16_deep_layers_of_many_mid_sized_jobs_take_one_64_row_tile():
    """Enough jobs to fill the chip and layers at least 1024 deep: 64-row tiles of 128
    columns (one per job up to 64 rows, two above, the second reading the weights
    from L2); ragged K and N, strips, and a round that mixes them with shallow layers."""
    deep = [dict(M=[33, 48, 64, 40][i % 4], dims=(1032, 904), acts=[[GELU, RELU, NONE][i % 3]]) for i in range(30)]
    deep += [dict(M=[64, 57][i % 2], dims=(1024, 1024), acts=[GELU], strip=True) for i in range(6)]
    outs, refs, launches = run_jobs(deep, salus.BF16)            # 30 x 8 + 6 x 8 column tiles >= 256
    assert launches == 1
    for o, r, j in zip(outs, refs, deep):
        assert np.isfinite(o).all() and norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))
    two_tiles = [dict(M=[65, 100, 128, 127][i % 4], dims=(1032, 520), acts=[[RELU, GELU][i % 2]]) for i in range(30)]
    outs, refs, launches = run_jobs(two_tiles, salus.BF16)       # K is no multiple of 64: not for the LDS-tiled kernel
    assert launches == 1
    for o, r, j in zip(outs, refs, two_tiles):
        assert np.isfinite(o).all() and norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))
    mixed = deep[:32] + [dict(M=50, dims=(40, 1000), acts=[RELU]) for i in range(8)]
    outs, refs, launches = run_jobs(mixed, salus.BF16)
    assert launches == 2                                          # deep and shallow layers of the same depth
    for o, r, j in zip(outs, refs, mixed):
        assert np.isfinite(o).all() and norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))


def test_bf16_mixed_batch_sizes_and_depths_in_one_packed_iteration():
    jobs = [dict(M=m, dims=(256, 1024, 256, 264), acts=[GELU, GELU, NONE]) for m in (1, 7, 16, 23, 32)]
    jobs += [dict(M=9, dims=(128, 136), acts=[RELU]), dict(M=32, dims=(64, 64, 64, 64, 64), acts=[RELU] * 3 + [NONE])]
    outs, refs, launches = run_jobs(jobs, salus.BF16)
    assert launches == 4                       # one launch per layer depth, not per job
    for o, r, j in zip(outs, refs, jobs):
        e = norm_rel_err(o, r)
        assert e < TOL_BF16 and e < TOL_BF16_TIGHT, (j, e)


@pytest.mark.parametrize("M", [128, 129, 191, 192, 200, 256, 257, 300, 515, 770])
def test_bf16_jobs_with_many_rows_take_the_tiled_kernel(M):
    """M >= 128 and K a multiple of 64: LDS-tiled kernels (128 x 256 tiles; 256 x 256
    from 192 rows), so these shapes cover several tiles, ragged row and column tails
    and K of one, two, three and sixteen slabs."""
    shapes = [(64, 8, NONE), (192, 264, RELU), (128, 520, GELU), (1024, 256, NONE), (64, 1000, GELU)]
    jobs = [dict(M=M, dims=(K, N), acts=[act]) for K, N, act in shapes]
    jobs.append(dict(M=5, dims=(192, 264), acts=[GELU]))         # small job of the same round
    jobs.append(dict(M=M, dims=(40, 72), acts=[RELU]))           # K not a multiple of 64: streamed
    outs, refs, launches = run_jobs(jobs, salus.BF16)
    assert launches == 3                                          # tiled + streaming (small job, big job), same layer depth
    for o, r, j in zip(outs, refs, jobs):
        assert np.isfinite(o).all(), j
        assert norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))


def test_bf16_tiled_kernel_hidden_layers_round_to_bf16():
    jobs = [dict(M=m, dims=(256, 512, 320, 264), acts=[GELU, RELU, NONE]) for m in (128, 333, 600)]
    jobs.append(dict(M=7, dims=(256, 512, 320, 264), acts=[GELU, RELU, NONE]))
    outs, refs, launches = run_jobs(jobs, salus.BF16)
    assert launches == 9                      # 128-row tiles, 256-row tiles and streaming per layer depth
    for o, r, j in zip(outs, refs, jobs):
        e = norm_rel_err(o, r)
        assert np.isfinite(o).all() and e < TOL_BF16 and e < TOL_BF16_TIGHT, (j, e)


def test_bf16_mid_sized_batches_go_tiled_when_the_round_fills_the_chip():
    """65..127 rows: tiled only if the round's tiled jobs make up at least 256 workgroups."""
    jobs = [dict(M=[65, 80, 100, 127][i % 4], dims=(64, 2048), acts=[[NONE, RELU, GELU][i % 3]]) for i in range(64)]
    outs, refs, launches = run_jobs(jobs, salus.BF16)
    assert launches == 1
    for o, r, j in zip(outs, refs, jobs):
        assert np.isfinite(o).all() and norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))
    outs, refs, launches = run_jobs(jobs[:8], salus.BF16)          # 64 workgroups: streamed instead
    assert launches == 1
    for o, r, j in zip(outs, refs, jobs):
        assert norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))


@pytest.mark.parametrize("M", [1, 9, 32, 70, 128, 300])
def test_bf16_strip_layout_gives_the_same_bits_as_row_major(M):
    """Weights stored in 128-column strips: same arithmetic in the same order, so
    the outputs equal the row-major ones bit for bit (and the oracle within tolerance)."""
    shapes = [(64, 128, NONE), (192, 384, RELU), (1024, 256, GELU), (40, 128, NONE), (264, 1024, GELU)]
    jobs = [dict(M=M, dims=(K, N), acts=[act]) for K, N, act in shapes]
    jobs.append(dict(M=M, dims=(256, 512, 384, 136), acts=[GELU, RELU, NONE]))     # last layer stays row-major
    plain, refs, _ = run_jobs(jobs, salus.BF16)
    strip, refs2, _ = run_jobs([dict(j, strip=True) for j in jobs], salus.BF16)
    for a, b, r, j in zip(plain, strip, refs, jobs):
        assert np.array_equal(a, b), j
        assert norm_rel_err(b, r) < TOL_BF16_TIGHT, j


def test_strip_layout_is_validated():
    dp = DevicePool(1 << 20, policy=salus.POLICY_PACK)
    a = dp.pool.lane_alloc(65536, 65536, 0, 1)[1]
    mk = lambda dtype, layers: salus.Pool.make_descs([dict(job=a, M=4, dtype=dtype, x_off=0, y_off=4096,
                                                           h_off=8192, layers=layers)])[0]
    assert dp.pool.grouped_forward(mk(salus.BF16, [(64, 128, 0, 0, salus.LAYOUT_STRIP128)])) == salus.OK
    assert dp.pool.grouped_forward(mk(salus.BF16, [(64, 64, 0, 0, salus.LAYOUT_STRIP128)])) == salus.EINVAL
    assert dp.pool.grouped_forward(mk(salus.F32, [(64, 128, 0, 0, salus.LAYOUT_STRIP128)])) == salus.EINVAL
    assert dp.pool.grouped_forward(mk(salus.BF16, [(64, 128, 0, 0, 7)])) == salus.EINVAL
    dp.close()


def test_more_jobs_than_one_launch_holds():
    jobs = [dict(M=1 + (i % 5), dims=(64, 72), acts=[NONE]) for i in range(70)]
    outs, refs, launches = run_jobs(jobs, salus.BF16)
    assert launches == 2
    for o, r in zip(outs, refs):
        assert norm_rel_err(o, r) < TOL_BF16_TIGHT


@pytest.mark.parametrize("M", [1, 8, 16, 19, 40, 64, 67])
def test_f32_ragged_shapes(M):
    jobs = [dict(M=M, dims=d, acts=a) for d, a in
            [((4, 4), [NONE]), ((20, 36), [RELU]), ((256, 256, 256), [RELU, NONE]),
             ((132, 68, 260), [GELU, NONE]), ((1024, 64), [NONE])]]
    outs, refs, launches = run_jobs(jobs, salus.F32)
    assert launches == 2
    for o, r, j in zip(outs, refs, jobs):
        assert np.isfinite(o).all(), j
        assert norm_rel_err(o, r) < TOL_F32, (j, norm_rel_err(o, r))


def test_f32_gelu_outputs_of_small_magnitude_and_in_the_negative_tail():
    """The float bound is relative to the largest output of a matrix, so GELU must
    be accurate relative to its own value: inputs of order 1e-3 (outputs ~ z / 2)
    and pre-activations that are all in [-6, -3.5], where 1 + erf is 1e-4 .. 1e-9
    and every output is below 1e-3 in magnitude."""
    jobs = [dict(M=19, dims=(256, 132), acts=[GELU], x_lo=-1e-3, x_hi=1e-3),
            dict(M=8, dims=(256, 256, 68), acts=[GELU, GELU], x_lo=-1e-3, x_hi=1e-3),
            dict(M=33, dims=(128, 260), acts=[GELU], x_lo=0.9, x_hi=1.0, w_scale=0.5, w_mean=-5.0),
            dict(M=16, dims=(64, 64), acts=[GELU], x_lo=0.99, x_hi=1.0, w_scale=0.05, w_mean=-4.0)]
    outs, refs, launches = run_jobs(jobs, salus.F32)
    for o, r, j in zip(outs, refs, jobs):
        assert np.isfinite(o).all(), j
        assert np.abs(r).max() < 2e-3, (j, np.abs(r).max())           # the case really is a small-output one
        assert norm_rel_err(o, r) < TOL_F32, (j, norm_rel_err(o, r))
    assert (refs[2] <= 0).all() and (refs[3] <= 0).all()              # all in the negative tail


def test_bf16_gelu_inputs_of_small_magnitude():
    """The bf16 kernels' erf approximation has an absolute error, scaled by the
    input: outputs of order 1e-3 still meet the tight relative bound."""
    jobs = [dict(M=m, dims=(256, 264), acts=[GELU], x_lo=-1e-3, x_hi=1e-3) for m in (7, 32, 64, 200)]
    outs, refs, launches = run_jobs(jobs, salus.BF16)
    for o, r, j in zip(outs, refs, jobs):
        assert np.abs(r).max() < 2e-3 and norm_rel_err(o, r) < TOL_BF16_TIGHT, (j, norm_rel_err(o, r))


def test_bf16_gelu_in_the_negative_tail():
    """Pre-activations that are all in [-6, -3.5]: every output is below 1e-3 in magnitude
    and the kernels' approximation of the normal tail, whose error is absolute (3e-7), is
    what decides the comparison.  It stays inside the bf16 bound relative to the largest
    output of the matrix (|z| * 3e-7 against 3.5 * 2.3e-4)."""
    jobs = [dict(M=33, dims=(128, 264), acts=[GELU], x_lo=0.9, x_hi=1.0, w_scale=0.5, w_mean=-5.0),
            dict(M=16, dims=(64, 64), acts=[GELU], x_lo=0.99, x_hi=1.0, w_scale=0.05, w_mean=-4.0),
            dict(M=200, dims=(128, 264), acts=[GELU], x_lo=0.9, x_hi=1.0, w_scale=0.5, w_mean=-5.0)]
    outs, refs, launches = run_jobs(jobs, salus.BF16)
    for o, r, j in zip(outs, refs, jobs):
        e = norm_rel_err(o, r)
        print("bf16 GELU tail", j["M"], "largest |ref|", np.abs(r).max(), "error", e)
        assert np.isfinite(o).all() and (r <= 0).all() and np.abs(r).max() < 2e-3, j
        assert e < TOL_BF16, (j, e)


def test_special_weights_bf16():
    """W = I copies the input, a single one at (k, n) moves column k to column n:
    catches a transposed or permuted operand independently of the oracle's GEMM."""
    K = 136
    dp = DevicePool(1 << 20, policy=salus.POLICY_PACK)
    w_offs, P, x_off, y_off, h_off, E = mlp_layout((K, K), 2, 16)
    st, jid = dp.pool.lane_alloc(P, E, 0, 2)
    q = dp.pool.job_query(jid)
    X = np.arange(16 * K, dtype=np.float32).reshape(16, K) % 251 - 125     # exact in bf16
    dp.write(q.lane_off + x_off, synth.f32_to_bf16_bits(X))
    items = [dict(job=jid, M=16, dtype=salus.BF16, x_off=x_off, y_off=y_off, h_off=h_off,
                  layers=[(K, K, 0, NONE)])]
    descs, keep = salus.Pool.make_descs(items)
    dp.write(q.persist_off, synth.f32_to_bf16_bits(np.eye(K, dtype=np.float32)))
    assert dp.pool.grouped_forward(descs, stream=dp.stream) == salus.OK
    assert np.array_equal(dp.read(q.lane_off + y_off, 16 * K * 4, np.float32).reshape(16, K), X)
    W = np.zeros((K, K), np.float32)
    W[3, 77] = 1.0
    W[130, 5] = 2.0
    dp.write(q.persist_off, synth.f32_to_bf16_bits(W))
    assert dp.pool.grouped_forward(descs, stream=dp.stream) == salus.OK
    Y = dp.read(q.lane_off + y_off, 16 * K * 4, np.float32).reshape(16, K)
    want = np.zeros_like(X)
    want[:, 77] = X[:, 3]
    want[:, 5] = 2 * X[:, 130]
    assert np.array_equal(Y, want)
    dp.close()


def test_forward_rejects_bad_descriptors():
    dp = DevicePool(1 << 20, policy=salus.POLICY_PACK, max_lanes=1)
    a = dp.pool.lane_alloc(65536, 65536, 0, 1)[1]
    b = dp.pool.lane_alloc(65536, 65536, 0, 1)[1]          # shares the only lane
    mk = lambda **kw: salus.Pool.make_descs([dict(dict(job=a, M=4, dtype=salus.BF16, x_off=0, y_off=4096,
                                                      h_off=8192, layers=[(64, 64, 0, 0)]), **kw)])
    ok, keep = mk()
    assert dp.pool.grouped_forward(ok) == salus.OK
    both, keep2 = salus.Pool.make_descs([dict(job=j, M=4, dtype=salus.BF16, x_off=0, y_off=4096, h_off=8192,
                                              layers=[(64, 64, 0, 0)]) for j in (a, b)])
    assert dp.pool.grouped_forward(both) == salus.EBUSY      # one lane runs one job at a time
    assert dp.pool.grouped_forward(mk(layers=[(64, 60, 0, 0)])[0]) == salus.EINVAL      # N not a multiple of 8
    assert dp.pool.grouped_forward(mk(layers=[(64, 64, 65536 - 64, 0)])[0]) == salus.EINVAL   # weights outside P
    assert dp.pool.grouped_forward(mk(y_off=65536 - 64)[0]) == salus.EINVAL             # output outside the lane
    assert dp.pool.grouped_forward(mk(y_off=0)[0]) == salus.EINVAL                      # x and y overlap
    assert dp.pool.grouped_forward(mk(M=0)[0]) == salus.EINVAL                          # a job without rows
    assert dp.pool.grouped_forward(ok, n=0) == salus.OK                                 # an empty round is legal
    launches = dp.pool.stats()["gemm_launches"]
    assert dp.pool.grouped_forward(ok, n=0) == salus.OK and dp.pool.stats()["gemm_launches"] == launches
    assert dp.pool.switch_out(a) == salus.OK
    assert dp.pool.grouped_forward(ok) == salus.ENOTRESIDENT
    dp.close()
