"""A packed round is only kernel launches with by-value arguments, so a caller
can record it in a HIP graph and replay it (launch-bound rounds: a handful of
tiles per layer).  The library records nothing but its own kernels: no memset
node, no allocation, no synchronisation.  Every replay is checked against the
oracle, with eager work between the replays."""
import numpy as np
import pytest
import torch

from oracle import dense
from paper_1902_04610_amd import salus, synth
from gpu_util import DevicePool, mlp_layout, norm_rel_err

pytestmark = pytest.mark.gpu


def test_the_fused_forward_refuses_to_be_recorded():
    # its counter sets alternate between launches; a replayed recording would reuse one
    dims, M = (64, 64, 64), 4
    w_offs, P, x_off, y_off, h_off, E = mlp_layout(dims, 2, M)
    dp = DevicePool((P + E + 4096 + 255) // 256 * 256, policy=salus.POLICY_PACK, fuse_depths=True)
    st, jid = dp.pool.lane_alloc(P, E, 0, 0)
    dp.buf.zero_()
    descs, keep = salus.Pool.make_descs([dict(job=jid, M=M, dtype=salus.BF16, x_off=x_off, y_off=y_off, h_off=h_off,
                                              layers=[(64, 64, w_offs[0], salus.ACT_RELU),
                                                      (64, 64, w_offs[1], salus.ACT_NONE)])])
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        rc = dp.pool.grouped_forward(descs, stream=side.cuda_stream)
    assert rc == salus.EINVAL and "graph" in dp.pool.last_error()
    assert dp.pool.grouped_forward(descs, stream=side.cuda_stream) == salus.OK      # eager is fine
    side.synchronize()
    assert dp.pool.fused_check() == salus.OK
    dp.close()


@pytest.mark.parametrize("dtype,fuse,static", [(salus.F32, False, False), (salus.BF16, False, False),
                                               (salus.F32, False, True), (salus.BF16, False, True)])
def test_a_recorded_round_replays_with_new_inputs(dtype, fuse, static):
    """static: the entry point that keeps the hidden activations in the library's
    own device array (what a caller under capture uses when it cannot allocate)."""
    esz = 4 if dtype == salus.F32 else 2
    dims, M, acts = (256, 256, 264), 8, [salus.ACT_RELU, salus.ACT_NONE]
    w_offs, P, x_off, y_off, h_off, E = mlp_layout(dims, esz, M)
    n_jobs = 3
    cap = (n_jobs * (P + E) + 4096 + 255) // 256 * 256
    dp = DevicePool(cap, policy=salus.POLICY_PACK, fuse_depths=fuse)
    rng = np.random.default_rng(21)
    jobs, W, items = [], [], []
    for _ in range(n_jobs):
        st, jid = dp.pool.lane_alloc(P, E, 0, 0)
        assert st == salus.OK
        q = dp.pool.job_query(jid)
        Ws = [(rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32) for K, N in zip(dims[:-1], dims[1:])]
        if dtype == salus.BF16:
            Ws = [synth.f32_to_bf16_bits(w) for w in Ws]
        for w, off in zip(Ws, w_offs):
            dp.write(q.persist_off + off, w)
        jobs.append(jid)
        W.append(Ws)
        items.append(dict(job=jid, M=M, dtype=dtype, x_off=x_off, y_off=y_off, h_off=h_off,
                          layers=[(K, N, off, a) for K, N, off, a in zip(dims[:-1], dims[1:], w_offs, acts)]))
    descs, keep = salus.Pool.make_descs(items)

    def put_inputs():
        X = []
        for jid in jobs:
            x = rng.uniform(-1, 1, (M, dims[0])).astype(np.float32)
            if dtype == salus.BF16:
                x = synth.f32_to_bf16_bits(x)
            q = dp.pool.job_query(jid)
            dp.write(q.lane_off + x_off, x)
            dp.write(q.lane_off + y_off, np.full((M, dims[-1]), np.nan, np.float32))
            X.append(x)
        return X

    def check(X, tag):
        fwd = dense.mlp_forward_f32 if dtype == salus.F32 else dense.mlp_forward_bf16
        for jid, x, Ws in zip(jobs, X, W):
            q = dp.pool.job_query(jid)
            y = dp.read(q.lane_off + y_off, M * dims[-1] * 4, np.float32).reshape(M, dims[-1])
            ref = fwd(x, Ws, acts)[-1]
            assert norm_rel_err(y, ref) < (1e-5 if dtype == salus.F32 else 2e-3), (tag, jid)

    forward = dp.pool.grouped_forward_static if static else dp.pool.grouped_forward
    side = torch.cuda.Stream()
    X = put_inputs()
    torch.cuda.synchronize()
    # one eager round on the side stream first (the fused path uploads its descriptors
    # then, so that the recorded round holds the forward launch only; the static variant
    # looks up its array's address at its first call on a device)
    assert forward(descs, stream=side.cuda_stream) == salus.OK
    side.synchronize()
    check(X, "eager")

    graph = torch.cuda.CUDAGraph()
    X = put_inputs()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        assert forward(descs, stream=side.cuda_stream) == salus.OK
    for replay in range(4):
        if replay:
            X = put_inputs()                       # eager copies between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check(X, f"replay {replay}")
        assert dp.pool.fused_check() == salus.OK
    dp.close()
