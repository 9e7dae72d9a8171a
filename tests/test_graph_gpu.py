"""The entry points only enqueue kernels on the caller's stream (no allocation, no synchronisation, no
memset), so a caller may record them into a HIP graph.  Captured once, replayed several times with new
input contents and eager work in between; every replay must equal the eager call bit for bit and agree
with the oracle."""
import numpy as np
import pytest
import torch

from _util import dev, to_np, rel_l2, TOL, pack_mask_np, masks_to_dev

pytestmark = pytest.mark.gpu


def _inputs(rng, N, L, bf16):
    g = (rng.standard_normal((N, L)) * 1e-3).astype(np.float32)
    recv = rng.random((N, L)) > 0.03
    recv[0] = True
    t = torch.from_numpy(g)
    return (t.bfloat16() if bf16 else t), pack_mask_np(recv)


@pytest.mark.parametrize("k,bf16", [(12, False), (16, True), (14, False), (15, True)])
def test_fused_path_in_a_graph(k, bf16):
    import paper_2310_06993_amd.binding as b
    import oracle
    N, L, seed = 4, 2 << k, 77
    rng = np.random.default_rng(1000 + k)
    fused = b.or_fused_path_bf16 if bf16 else b.or_fused_path
    dt = torch.bfloat16 if bf16 else torch.float32
    g = torch.empty((N, L), dtype=dt, device=dev())
    m = torch.empty((N, L // 32), dtype=torch.int32, device=dev())
    out = torch.empty(L, dtype=dt, device=dev())
    cnt = torch.empty(L, dtype=torch.uint8, device=dev())
    nws = b.or_workspace_bytes(L, k)
    ws = torch.empty(nws, dtype=torch.uint8, device=dev()) if nws else None
    total = torch.zeros(1, dtype=torch.int64, device=dev())

    g0, m0 = _inputs(rng, N, L, bf16)
    g.copy_(g0)
    m.copy_(masks_to_dev(m0))
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fused(g, m, N, L, k, seed, 0, out, cnt, ws)
        b.or_received_total(cnt, L, total)      # clears its accumulator with a kernel, not a memset
    for rep in range(4):
        gi, mi = _inputs(rng, N, L, bf16)
        g.copy_(gi)
        m.copy_(masks_to_dev(mi))
        out.fill_(float("nan"))
        cnt.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got, got_cnt, got_total = to_np(out).copy(), to_np(cnt).copy(), int(total.item())
        # the same call eagerly, into other buffers
        out2, cnt2 = torch.empty_like(out), torch.empty_like(cnt)
        fused(g, m, N, L, k, seed, 0, out2, cnt2, ws)
        torch.cuda.synchronize()
        assert np.array_equal(got, to_np(out2)) and np.array_equal(got_cnt, to_np(cnt2)), rep
        want, wcnt = oracle.fused_path(to_np(g), mi, k, seed, 0)
        assert np.array_equal(got_cnt, wcnt) and got_total == int(wcnt.sum())
        assert rel_l2(got, want) <= TOL["bf16" if bf16 else "f32"]


def test_three_calls_in_a_graph():
    import paper_2310_06993_amd.binding as b
    import oracle
    N, k, seed = 4, 11, 5
    L = 6 << k
    rng = np.random.default_rng(42)
    grad = torch.empty(N * L, device=dev())          # one worker's whole gradient, encoded in one call
    shards = torch.empty((N, L), device=dev())       # what the owner of shard 0 received
    m = torch.empty((N, L // 32), dtype=torch.int32, device=dev())
    enc = torch.empty(N * L, device=dev())
    total = torch.empty(L, device=dev())
    cnt = torch.empty(L, dtype=torch.uint8, device=dev())
    out = torch.empty(L, device=dev())
    graph = torch.cuda.CUDAGraph()
    grad.normal_()
    shards.normal_()
    m.fill_(-1)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        b.or_rht_encode(grad, N * L, k, seed, enc)
        b.or_masked_reduce(shards, m, N, L, total, cnt)
        b.or_finalize_decode(total, cnt, L, k, seed, 0, out)
    for rep in range(3):
        gi = (rng.standard_normal(N * L) * 1e-3).astype(np.float32)
        si = (rng.standard_normal((N, L)) * 1e-3).astype(np.float32)
        recv = rng.random((N, L)) > 0.05
        recv[0] = True
        mi = pack_mask_np(recv)
        grad.copy_(torch.from_numpy(gi))
        shards.copy_(torch.from_numpy(si))
        m.copy_(masks_to_dev(mi))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert rel_l2(to_np(enc), oracle.rht_encode(gi, k, seed)) <= TOL["f32"]
        wsum, wcnt = oracle.masked_reduce(si, mi)
        assert np.array_equal(to_np(cnt), wcnt) and rel_l2(to_np(total), wsum) <= TOL["f32"]
        want = oracle.rht_decode(oracle.finalize(wsum, wcnt), L, k, seed, 0)
        assert rel_l2(to_np(out), want) <= TOL["f32"]
