"""Synthetic stand-in for the paper's Hadamard study (Sec. 5.3, accuracy with and without the transform
at 1 / 5 / 10 % dropped entries; Sec. 3.3 dispersal) and for its loss-propagation comparison of Ring, parameter
server and TAR (Sec. 5.3): with tail drops the transform spreads the loss
over every entry of a block instead of concentrating it on the entries that went missing.  Runs the
library both ways (or_fused_path vs or_masked_reduce + or_finalize) on the GPU; no training involved."""
import numpy as np
import pytest
import torch

from _util import dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("loss", [0.01, 0.05, 0.10])
def test_tail_drops_with_and_without_transform(loss):
    import paper_2310_06993_amd.binding as b
    import oracle
    from _util import to_np, rel_l2, TOL
    N, k = 8, 12
    L = 64 << k
    gen = torch.Generator(device=dev()).manual_seed(int(loss * 1000))
    g = torch.randn((N, L), device=dev(), generator=gen) * 1e-3
    truth = g.double().mean(dim=0)
    # every worker but the owner loses the last `loss` fraction of each block-sized packet train:
    # a tail drop per block, the pattern the paper's Fig. 8 motivates
    m = torch.full((N, L // 32), -1, dtype=torch.int32, device=dev())
    words_per_block = (1 << k) // 32
    lost_words = max(1, int(round(words_per_block * loss * N / (N - 1))))
    mv = m.view(N, L >> k, words_per_block)
    mv[1:, :, words_per_block - lost_words:] = 0
    out = torch.empty(L, device=dev())
    cnt = torch.empty(L, dtype=torch.uint8, device=dev())
    b.or_fused_path(g, m, N, L, k, 7, 0, out, cnt)
    total = torch.empty(L, device=dev())
    b.or_masked_reduce(g, m, N, L, total, cnt)
    plain = torch.empty(L, device=dev())
    b.or_finalize(total, cnt, L, plain)
    # both routes against the oracle first: the figures below are then properties of the method, not of this build
    gh, mh = to_np(g), to_np(m)
    want, wcnt = oracle.fused_path(gh, mh, k, 7, 0)
    assert np.array_equal(to_np(cnt), wcnt) and rel_l2(to_np(out), want) <= TOL["f32"]
    wsum, wcnt2 = oracle.masked_reduce(gh, mh)
    assert np.array_equal(wcnt2, wcnt) and rel_l2(to_np(plain), oracle.finalize(wsum, wcnt2)) <= TOL["f32"]
    err_ht = (out.double() - truth).abs()
    err_plain = (plain.double() - truth).abs()
    lost = 1.0 - float(cnt.float().mean()) / N
    assert abs(lost - loss) < 0.35 * loss + 0.004
    # without the transform the entries in the tail fall back to the owner's own gradient: large error
    # there, none elsewhere; with it the same energy is spread thinly over whole blocks
    # worst entry: the spread error has about sqrt(loss) of the concentrated one's scale
    assert float(err_plain.max()) > 0.6 / np.sqrt(loss) * float(err_ht.max())
    tiny = 1e-8   # fp32 rounding of the mean itself is ~1e-11
    assert float((err_plain < tiny).double().mean()) > 0.8 and float((err_ht < tiny).double().mean()) < 0.05
    mse_ht, mse_plain = float((err_ht ** 2).mean()), float((err_plain ** 2).mean())
    assert 0.3 < mse_ht / mse_plain < 3.0
    # the estimate stays centred (unbiased): mean signed error is far below the typical error
    assert abs(float((out.double() - truth).mean())) < 0.05 * float(err_ht.mean() + 1e-30)
    # the figures themselves (shown with `pytest -s`; the paper's own study, Sec. 5.3, reports accuracy of a trained
    # model, which needs its dataset: these synthetic figures have no counterpart there -- parity unpinned)
    print("\n[tail drops %4.1f %%] MSE with transform %.3e, without %.3e; worst entry with %.3e, without %.3e; "
          "entries off by more than 1e-8: with %.1f %%, without %.1f %%"
          % (100 * lost, mse_ht, mse_plain, float(err_ht.max()), float(err_plain.max()),
             100 * float((err_ht >= tiny).double().mean()), 100 * float((err_plain >= tiny).double().mean())))


def test_255_workers_and_counts(b_or=None):
    import paper_2310_06993_amd.binding as b
    import oracle
    from _util import pack_mask_np, masks_to_dev, to_np, rel_l2, TOL
    N, k = 255, 10
    L = 2 << k
    rng = np.random.default_rng(255)
    g = (rng.standard_normal((N, L)) * 1e-3).astype(np.float32)
    recv = rng.random((N, L)) > 0.02
    recv[:, 100:164] = True          # entries every worker delivered: count 255
    masks = pack_mask_np(recv)
    out = torch.empty(L, device=dev())
    cnt = torch.empty(L, dtype=torch.uint8, device=dev())
    b.or_fused_path(torch.from_numpy(g).to(dev()), masks_to_dev(masks), N, L, k, 3, 0, out, cnt)
    want, wcnt = oracle.fused_path(g, masks, k, 3, 0)
    assert np.array_equal(to_np(cnt), wcnt) and int(wcnt.max()) == 255
    assert rel_l2(to_np(out), want) <= TOL["f32"]


def test_loss_propagation_ring_vs_ps_vs_direct():
    """Synthetic stand-in for the topology comparison of Sec. 5.3 (Ring has several times the MSE of TAR at
    the same loss; Sec. 3.1.1 gives the reason: in a ring the partial aggregate travels hop by hop, so one
    lost packet takes with it everything aggregated so far, while TAR's owner hears from every peer
    directly).  Same per-transfer packet loss for both; the ring is emulated, generously, with the
    count-carrying pair reduction (a hop whose packet is lost restarts from the receiver's own entries).
    Every aggregate is checked against the oracle; the ordering of the errors is the property."""
    import paper_2310_06993_amd.binding as b
    import oracle
    from _util import pack_mask_np, masks_to_dev, to_np, rel_l2, TOL
    N, L, packet, p = 8, 1 << 20, 256, 0.05
    rng = np.random.default_rng(2310)
    g = (rng.standard_normal((N, L)) * 1e-3).astype(np.float32)
    truth = g.astype(np.float64).mean(axis=0)

    def arrivals(rows):
        a = rng.random((rows, L // packet)) >= p
        return np.repeat(a, packet, axis=1)

    # TAR, first stage at the owner (node 0): N - 1 direct transfers, the owner's own shard is local
    recv = arrivals(N)
    recv[0] = True
    m_tar = pack_mask_np(recv)
    gd = torch.from_numpy(g).to(dev())
    total = torch.empty(L, device=dev())
    cnt = torch.empty(L, dtype=torch.uint8, device=dev())
    mean_tar = torch.empty(L, device=dev())
    b.or_masked_reduce(gd, masks_to_dev(m_tar), N, L, total, cnt)
    b.or_finalize(total, cnt, L, mean_tar)
    w_total, w_cnt = oracle.masked_reduce(g, m_tar)
    assert np.array_equal(to_np(cnt), w_cnt) and rel_l2(to_np(total), w_total) <= TOL["f32"]
    assert rel_l2(to_np(mean_tar), oracle.finalize(w_total, w_cnt)) <= TOL["f32"]

    # Ring: the partial for shard 0 starts at node 1 and visits 2, 3, ..., N-1, 0
    ones = np.ones((1, L), bool)
    one_count = torch.ones(L, dtype=torch.uint8, device=dev())
    part_sum, part_cnt = gd[1].clone(), one_count.clone()
    o_sum, o_cnt = g[1].copy(), np.ones(L, np.uint8)
    for node in list(range(2, N)) + [0]:
        m = pack_mask_np(np.concatenate([arrivals(1), ones]))
        sums = torch.stack([part_sum, gd[node]])
        counts = torch.stack([part_cnt, one_count])
        new_sum, new_cnt = torch.empty(L, device=dev()), torch.empty(L, dtype=torch.uint8, device=dev())
        b.or_masked_reduce_pairs(sums, counts, masks_to_dev(m), 2, L, new_sum, new_cnt)
        o_sum, o_cnt = oracle.masked_reduce_pairs(np.stack([o_sum, g[node]]), np.stack([o_cnt, np.ones(L, np.uint8)]), m)
        assert np.array_equal(to_np(new_cnt), o_cnt) and rel_l2(to_np(new_sum), o_sum) <= TOL["f32"]
        part_sum, part_cnt = new_sum, new_cnt
    mean_ring = torch.empty(L, device=dev())
    b.or_finalize(part_sum, part_cnt, L, mean_ring)
    assert rel_l2(to_np(mean_ring), oracle.finalize(o_sum, o_cnt)) <= TOL["f32"]

    # Parameter server: the owner of the WHOLE gradient hears from all N - 1 workers at once, every flow N times as
    # long as a TAR shard transfer.  What separates it from TAR on a real network is the loss that this incast
    # causes; a one-GPU model cannot derive that, so it is an input here: `incast` times the per-transfer loss.
    incast = 3.0
    recv_ps = np.repeat(rng.random((N, L // packet)) >= incast * p, packet, axis=1)
    recv_ps[0] = True
    m_ps = pack_mask_np(recv_ps)
    mean_ps = torch.empty(L, device=dev())
    b.or_masked_reduce(gd, masks_to_dev(m_ps), N, L, total, cnt)
    b.or_finalize(total, cnt, L, mean_ps)
    w_total, w_cnt = oracle.masked_reduce(g, m_ps)
    assert np.array_equal(to_np(cnt), w_cnt) and rel_l2(to_np(mean_ps), oracle.finalize(w_total, w_cnt)) <= TOL["f32"]

    mse_tar = float(((to_np(mean_tar).astype(np.float64) - truth) ** 2).mean())
    mse_ring = float(((to_np(mean_ring).astype(np.float64) - truth) ** 2).mean())
    mse_ps = float(((to_np(mean_ps).astype(np.float64) - truth) ** 2).mean())
    # expected contributions lost per entry: (N-1) p directly, about p N (N-1) / 2 along the ring
    assert mse_ring > 2.5 * mse_tar > 0
    assert mse_ring > mse_ps > 1.5 * mse_tar          # the paper's order: Ring > PS > TAR (14.55 / 9.92 / 2.47)
    assert int(part_cnt.min()) >= 1 and int(cnt.min()) >= 1
    # The paper's three values come from its cluster's loss process and a 500 M-entry tensor; these come from iid
    # packet loss on synthetic data -- only the order and the rough ratios are comparable (parity unpinned).
    print("\n[loss propagation, N = %d, %.0f %% packet loss per transfer, PS incast factor %.0f] MSE ring %.3e, "
          "parameter server %.3e, TAR %.3e; ring / TAR = %.2f, PS / TAR = %.2f (paper: 5.9 and 4.0)"
          % (N, 100 * p, incast, mse_ring, mse_ps, mse_tar, mse_ring / mse_tar, mse_ps / mse_tar))
