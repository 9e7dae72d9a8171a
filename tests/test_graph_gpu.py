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


def test_batched_monitored_and_static_calls_in_a_graph():
    """The batched fused call with its per-bucket arrival totals (zeroed by a kernel, not a memset) and the call
    with the static workspace (blocks of 2^16: sign stream, hand-over flags and slots all live in the library's
    array) recorded once and replayed with new inputs."""
    import paper_2310_06993_amd.binding as b
    import oracle
    N, seed = 4, 31
    rng = np.random.default_rng(77)
    k1, lens = 12, [3 << 12, 0, 5 << 12, 2 << 12]
    k2, L2 = 16, 12 << 16
    g1 = [torch.empty((N, L), device=dev()) for L in lens]
    m1 = [torch.empty((N, L // 32), dtype=torch.int32, device=dev()) for L in lens]
    o1 = [torch.empty(L, device=dev()) for L in lens]
    c1 = [torch.empty(L, dtype=torch.uint8, device=dev()) for L in lens]
    totals = torch.empty(len(lens), dtype=torch.int64, device=dev())
    arr = b.make_buckets([(g1[j], m1[j], o1[j], c1[j], lens[j], seed + j, 0) for j in range(len(lens))])
    g2 = torch.empty((N, L2), dtype=torch.bfloat16, device=dev())
    m2 = torch.empty((N, L2 // 32), dtype=torch.int32, device=dev())
    o2 = torch.empty(L2, dtype=torch.bfloat16, device=dev())
    c2 = torch.empty(L2, dtype=torch.uint8, device=dev())
    # first call outside the capture: it looks the static array's address up
    g2.zero_(); m2.fill_(-1)
    b.or_fused_path_bf16_static(g2, m2, N, L2, k2, seed, 0, o2, c2)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        b.or_fused_path_batched_monitored(arr, len(lens), N, k1, False, totals)
        b.or_fused_path_bf16_static(g2, m2, N, L2, k2, seed, 0, o2, c2)
    for rep in range(3):
        ins1 = [_inputs(rng, N, L, False) for L in lens]
        for j, (gi, mi) in enumerate(ins1):
            g1[j].copy_(gi); m1[j].copy_(masks_to_dev(mi))
        gi2, mi2 = _inputs(rng, N, L2, True)
        g2.copy_(gi2); m2.copy_(masks_to_dev(mi2))
        totals.fill_(-5); o2.fill_(float("nan")); c2.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        tot = totals.cpu().numpy()
        for j, (gi, mi) in enumerate(ins1):
            if lens[j] == 0:
                assert tot[j] == 0
                continue
            want, wcnt = oracle.fused_path(gi.numpy(), mi, k1, seed + j, 0)
            assert np.array_equal(to_np(c1[j]), wcnt) and int(tot[j]) == int(wcnt.sum()), (rep, j)
            assert rel_l2(to_np(o1[j]), want) <= TOL["f32"], (rep, j)
        want, wcnt = oracle.fused_path(to_np(g2), mi2, k2, seed, 0)
        assert np.array_equal(to_np(c2), wcnt), rep
        assert rel_l2(to_np(o2), want) <= TOL["bf16"], rep
