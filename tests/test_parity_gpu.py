"""HIP path vs CPU oracle, element by element, on seeded inputs (sizes the oracle does in seconds).

fp32 results must agree to a relative L2 error of 1e-6, bf16 results to 1e-2; sign draws, masks
and received counts must agree bit for bit.
"""
import numpy as np
import pytest
import torch

from _util import TOL, as_f64, dev, masks_to_dev, pack_mask_np, rel_l2, to_np

pytestmark = pytest.mark.gpu

ALL_K = list(range(5, 17))


@pytest.fixture(scope="module")
def b():
    import paper_2310_06993_amd.binding as binding
    assert torch.cuda.is_available()
    return binding


def _bf16_bits(x32: np.ndarray) -> np.ndarray:
    return to_np(torch.from_numpy(x32).to(torch.bfloat16))


def _dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16).copy()).to(dev()).view(torch.bfloat16)


def _sizes(k):
    """Lengths that span several tiles and end in a ragged block."""
    B = 1 << k
    tile = max(B, 1024) if k <= 14 else 1 << 14
    return [B * 3 - 5, max(3 * tile, 2 * B) + B + 17]


# ------------------------------------------------------------------ encode / decode
@pytest.mark.parametrize("k", ALL_K)
def test_encode_decode_fp32(b, orc, k):
    B = 1 << k
    rng = np.random.default_rng(k)
    for n in _sizes(k):
        seed, base = 1000 + k, max(B, 128) * 3
        x = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        n_pad = b.or_padded_len(n, k)
        assert n_pad == orc.padded_len(n, k)
        xd = torch.from_numpy(x).to(dev())
        enc = torch.full((n_pad,), float("nan"), device=dev())
        b.or_rht_encode_at(xd, n, k, seed, base, enc)
        want = orc.rht_encode(x, k, seed, base)
        assert rel_l2(to_np(enc), want) <= TOL["f32"], (k, n)
        y = (rng.standard_normal(n_pad) * 1e-3).astype(np.float32)
        dec = torch.full((n,), float("nan"), device=dev())
        b.or_rht_decode_at(torch.from_numpy(y).to(dev()), n, k, seed, base, dec)
        assert rel_l2(to_np(dec), orc.rht_decode(y, n, k, seed, base)) <= TOL["f32"], (k, n)
        # base_index 0 entry points
        if n == _sizes(k)[0]:
            b.or_rht_encode(xd, n, k, seed, enc)
            assert rel_l2(to_np(enc), orc.rht_encode(x, k, seed, 0)) <= TOL["f32"]
            b.or_rht_decode(enc.clone(), n, k, seed, dec)
            assert rel_l2(to_np(dec), x) <= 2 * TOL["f32"]


@pytest.mark.parametrize("k", [5, 8, 10, 11, 12, 13, 14, 15, 16])
def test_encode_decode_bf16(b, orc, k):
    B = 1 << k
    rng = np.random.default_rng(50 + k)
    n = _sizes(k)[1]
    seed, base = 77, max(B, 128)
    x = _bf16_bits((rng.standard_normal(n) * 1e-4).astype(np.float32))
    n_pad = b.or_padded_len(n, k)
    enc = torch.zeros(n_pad, dtype=torch.bfloat16, device=dev())
    b.or_rht_encode_bf16(_dev_bf16(x), n, k, seed, base, enc)
    want = orc.rht_encode(x, k, seed, base)
    assert rel_l2(to_np(enc), want) <= TOL["bf16"]
    # stricter: the two may differ only where fp32 vs fp64 arithmetic straddles a bf16 rounding boundary
    assert (to_np(enc) != want).mean() < 0.02
    y = (rng.standard_normal(n_pad) * 1e-4).astype(np.float32)
    dec = torch.zeros(n, dtype=torch.bfloat16, device=dev())
    b.or_rht_decode_bf16(torch.from_numpy(y).to(dev()), n, k, seed, base, dec)
    want = orc.rht_decode(y, n, k, seed, base, out_dtype=np.uint16)
    assert rel_l2(to_np(dec), want) <= TOL["bf16"]
    assert (to_np(dec) != want).mean() < 0.02


@pytest.mark.parametrize("k", [6, 10, 12, 14, 16])
def test_sign_draws_are_bit_exact(b, orc, k):
    # decode of sqrt(B) * e_0 in every block is exactly the sign vector (even k: all values exact)
    B = 1 << k
    n = 5 * B if k < 14 else 2 * B
    seed, base = (0xABCDEF << 24) + k, 7 * max(B, 128)
    agg = np.zeros(n, np.float32)
    agg[::B] = np.sqrt(B)
    out = torch.empty(n, device=dev())
    b.or_rht_decode_at(torch.from_numpy(agg).to(dev()), n, k, seed, base, out)
    want = 1.0 - 2.0 * orc.sign_bits(seed, base, n).astype(np.float32)
    assert np.array_equal(to_np(out), want)


def test_sign_stream_beyond_2_to_32(b, orc):
    k, base, seed = 12, (1 << 33) + (1 << 12) * 5, 99
    n = 1 << 13
    agg = np.zeros(n, np.float32)
    agg[:: 1 << k] = 64.0
    out = torch.empty(n, device=dev())
    b.or_rht_decode_at(torch.from_numpy(agg).to(dev()), n, k, seed, base, out)
    assert np.array_equal(to_np(out), 1.0 - 2.0 * orc.sign_bits(seed, base, n).astype(np.float32))


@pytest.mark.parametrize("k", [6, 8, 10, 12, 14, 16])
def test_integer_round_trip_is_bit_exact(b, k):
    # H(Hx) = Bx: with small integers and even k every intermediate is exact in fp32
    B = 1 << k
    n = 3 * B
    x = torch.randint(-3, 4, (n,), device=dev(), generator=torch.Generator(device=dev()).manual_seed(k)).float()
    enc = torch.empty(n, device=dev())
    dec = torch.empty(n, device=dev())
    b.or_rht_encode(x, n, k, 5, enc)
    b.or_rht_decode(enc, n, k, 5, dec)
    assert torch.equal(dec, x)
    # Parseval on the GPU result
    assert abs(float(enc.double().norm() / x.double().norm()) - 1.0) < 1e-6
    # in place is allowed when the length is whole blocks
    y = x.clone()
    b.or_rht_encode(y, n, k, 5, y)
    assert torch.equal(y, enc)
    b.or_rht_decode(y, n, k, 5, y)
    assert torch.equal(y, x)


# ------------------------------------------------------------------ aggregation
@pytest.mark.parametrize("N,L", [(1, 32), (3, 96), (4, 32 * 257), (8, 32 * 1000 + 64), (16, 4096 * 3), (255, 64)])
@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_masked_reduce(b, orc, N, L, kind):
    rng = np.random.default_rng(N * 1000 + L)
    x = rng.standard_normal((N, L)).astype(np.float32)
    recv = rng.random((N, L)) > 0.2
    masks = pack_mask_np(recv)
    total = torch.empty(L, device=dev())
    count = torch.empty(L, dtype=torch.uint8, device=dev())
    if kind == "f32":
        shards = x
        poisoned = np.where(recv, x, np.nan).astype(np.float32)   # lost slots hold NaN: never read
        b.or_masked_reduce(torch.from_numpy(poisoned).to(dev()), masks_to_dev(masks), N, L, total, count)
    else:
        shards = _bf16_bits(x)
        poisoned = np.where(recv, shards, 0x7FC0).astype(np.uint16)
        b.or_masked_reduce_bf16(_dev_bf16(poisoned), masks_to_dev(masks), N, L, total, count)
    want_sum, want_count = orc.masked_reduce(shards, masks)
    assert np.array_equal(to_np(count), want_count)
    assert np.isfinite(to_np(total)).all()
    assert rel_l2(to_np(total), want_sum) <= TOL["f32"]


@pytest.mark.parametrize("k", [5, 9, 10, 12, 14, 16])
def test_finalize_decode(b, orc, k):
    B = 1 << k
    n = _sizes(k)[0]
    n_pad = b.or_padded_len(n, k)
    rng = np.random.default_rng(k + 300)
    total = rng.standard_normal(n_pad).astype(np.float32)
    count = rng.integers(0, 9, n_pad).astype(np.uint8)
    seed, base = 31, 2 * max(B, 128)
    want = orc.rht_decode(orc.finalize(total, count), n, k, seed, base)
    out = torch.empty(n, device=dev())
    b.or_finalize_decode(torch.from_numpy(total).to(dev()), torch.from_numpy(count).to(dev()), n, k, seed, base, out)
    assert rel_l2(to_np(out), want) <= TOL["f32"]
    outh = torch.empty(n, dtype=torch.bfloat16, device=dev())
    b.or_finalize_decode_bf16(torch.from_numpy(total).to(dev()), torch.from_numpy(count).to(dev()), n, k, seed, base,
                              outh)
    assert rel_l2(to_np(outh), orc.rht_decode(orc.finalize(total, count), n, k, seed, base, out_dtype=np.uint16)) \
        <= TOL["bf16"]


def _workspace(b, L, k):
    nbytes = b.or_workspace_bytes(L, k)
    return torch.empty(nbytes, dtype=torch.uint8, device=dev()) if nbytes else None


@pytest.mark.parametrize("k,N,blocks", [(5, 3, 70), (7, 4, 9), (10, 4, 5), (11, 8, 3), (12, 8, 3), (13, 2, 2),
                                        (14, 5, 2), (15, 3, 2), (16, 4, 2)])
@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_reduce_decode_and_fused(b, orc, k, N, blocks, kind):
    B = 1 << k
    L = blocks * B
    rng = np.random.default_rng(k * 100 + N)
    raw32 = (rng.standard_normal((N, L)) * 1e-3).astype(np.float32)
    recv = rng.random((N, L)) > 0.03
    recv[:, 5 * 32: 6 * 32] = False          # a word nobody delivered: count 0 -> mean 0
    recv[1 % N, : L // 2] = rng.random(L // 2) > 0.5
    masks = pack_mask_np(recv)
    md = masks_to_dev(masks)
    seed, base = 4242 + k, 3 * max(B, 128)
    ws = _workspace(b, L, k)
    count = torch.empty(L, dtype=torch.uint8, device=dev())
    if kind == "f32":
        raw = raw32
        want, want_count = orc.fused_path(raw, masks, k, seed, base)
        out = torch.empty(L, device=dev())
        b.or_fused_path(torch.from_numpy(raw).to(dev()), md, N, L, k, seed, base, out, count, ws)
        assert np.array_equal(to_np(count), want_count)
        assert rel_l2(to_np(out), want) <= TOL["f32"]
        # encoded shards in, decoded shard out; NaN in the slots that never arrived
        enc = np.stack([orc.rht_encode(raw[i], k, seed, base) for i in range(N)])
        encd = torch.from_numpy(np.where(recv, enc, np.nan).astype(np.float32)).to(dev())
        out2 = torch.empty(L, device=dev())
        count.zero_()
        b.or_reduce_decode(encd, md, N, L, k, seed, base, out2, count, ws)
        assert np.array_equal(to_np(count), want_count)
        assert rel_l2(to_np(out2), want) <= TOL["f32"]
        # count_out is optional
        out3 = torch.empty(L, device=dev())
        b.or_fused_path(torch.from_numpy(raw).to(dev()), md, N, L, k, seed, base, out3, None, ws)
        assert torch.equal(out3, out)
    else:
        raw = _bf16_bits(raw32)
        want, want_count = orc.fused_path(raw, masks, k, seed, base)
        out = torch.empty(L, dtype=torch.bfloat16, device=dev())
        b.or_fused_path_bf16(_dev_bf16(raw), md, N, L, k, seed, base, out, count, ws)
        assert np.array_equal(to_np(count), want_count)
        assert rel_l2(to_np(out), want) <= TOL["bf16"]
        enc = np.stack([orc.rht_encode(raw[i], k, seed, base) for i in range(N)])
        out2 = torch.empty(L, dtype=torch.bfloat16, device=dev())
        b.or_reduce_decode_bf16(_dev_bf16(np.where(recv, enc, 0x7FC0).astype(np.uint16)), md, N, L, k, seed, base,
                                out2, count, ws)
        assert np.array_equal(to_np(count), want_count)
        assert rel_l2(to_np(out2), want) <= TOL["bf16"]
        # with the encoded shards given, only fp32-vs-fp64 summation differs: much tighter than 1e-2
        assert (to_np(out2) != want).mean() < 0.02


@pytest.mark.parametrize("k,N,blocks", [(16, 1, 1), (15, 9, 3), (16, 2, 3), (12, 1, 2), (14, 17, 1), (12, 2, 1),
                                        (12, 5, 3), (11, 4, 5), (9, 7, 11), (12, 16, 2)])
def test_fused_worker_counts_and_64_bit_seeds(b, orc, k, N, blocks):
    """One worker, odd worker counts, a seed with high bits set, a base index beyond 2^32."""
    L = blocks << k
    rng = np.random.default_rng(9000 + 17 * k + N)
    raw = (rng.standard_normal((N, L)) * 1e-3).astype(np.float32)
    recv = rng.random((N, L)) > 0.04
    masks = pack_mask_np(recv)
    seed, base = 0xF00DFACE12345678, (1 << 33) + 5 * max(1 << k, 128)
    want, want_count = orc.fused_path(raw, masks, k, seed, base)
    out = torch.empty(L, device=dev())
    count = torch.empty(L, dtype=torch.uint8, device=dev())
    b.or_fused_path(torch.from_numpy(raw).to(dev()), masks_to_dev(masks), N, L, k, seed, base, out, count,
                    _workspace(b, L, k))
    assert np.array_equal(to_np(count), want_count)
    assert rel_l2(to_np(out), want) <= TOL["f32"]


@pytest.mark.parametrize("k,N,blocks", [(16, 1, 1), (16, 2, 9), (16, 9, 17), (15, 1, 3), (15, 9, 4), (16, 255, 1), (15, 64, 2)])
def test_fused_bf16_large_blocks_worker_counts_and_loss_patterns(b, orc, k, N, blocks):
    """The bf16 kernel for blocks of 2^15 / 2^16 entries decides per worker whether anything of its two output tiles
    was lost: workers with nothing lost, with single entries lost, with a whole tile lost and with everything lost
    side by side; one worker, odd and large worker counts, more blocks than a group of 8 (the placement of the
    workgroups of a block), a seed with high bits set and a base index beyond 2^32."""
    B, T = 1 << k, 1 << 14
    L = blocks * B
    rng = np.random.default_rng(7000 + 31 * k + N)
    raw = _bf16_bits((rng.standard_normal((N, L)) * 1e-4).astype(np.float32))
    recv = np.ones((N, L), bool)
    for i in range(N):
        kind = i % 5
        if kind == 1:                                   # scattered single entries
            recv[i] = rng.random(L) > 0.01
        elif kind == 2:                                 # one whole tile, in every second block
            for blk in range(0, blocks, 2):
                t = (i // 5 + blk) % (B // T)
                recv[i, blk * B + t * T: blk * B + (t + 1) * T] = False
        elif kind == 3:                                 # a 512-entry packet here and there
            ok = rng.random(L // 512) > 0.03
            recv[i] = np.repeat(ok, 512)
        elif kind == 4 and N > 4:                       # nothing of this worker arrived
            recv[i] = False
    masks = pack_mask_np(recv)
    seed, base = 0xF00DFACE12345678, (1 << 33) + 5 * B
    want, want_count = orc.fused_path(raw, masks, k, seed, base)
    out = torch.full((L,), float("nan"), dtype=torch.bfloat16, device=dev())
    count = torch.full((L,), 77, dtype=torch.uint8, device=dev())
    total = torch.full((1,), -1, dtype=torch.int64, device=dev())
    gd, md, ws = _dev_bf16(raw), masks_to_dev(masks), _workspace(b, L, k)   # (the descriptor holds plain addresses)
    arr = b.make_buckets([(gd, md, out, count, L, seed, base)])
    b.or_fused_path_batched_monitored(arr, 1, N, k, True, total, ws)
    assert np.array_equal(to_np(count), want_count)
    assert int(total.item()) == int(want_count.sum(dtype=np.int64)) == int(recv.sum())
    assert rel_l2(to_np(out), want) <= TOL["bf16"]
    # block by block as well: a block with a wrong factor would hide in the total
    for blk in range(blocks):
        sl = slice(blk * B, (blk + 1) * B)
        assert rel_l2(to_np(out[sl]), want[sl]) <= TOL["bf16"], blk
    assert (to_np(out) != want).mean() < 0.05          # bf16 values: almost all identical, the rest one step apart


def test_three_calls_equal_fused(b, orc):
    from paper_2310_06993_amd import workloads as wl
    cfg = wl.CONFIGS["tiny"]
    N, L, k = cfg.workers, cfg.shard_len(), cfg.block_log2
    assert (N, L, k) == (4, 16384, 10)
    g = wl.make_grads(cfg, dev(), shard=1)
    m = wl.make_masks(cfg, dev(), shard=1)
    seed, base = cfg.seed, 1 * L
    enc = torch.empty((N, L), device=dev())
    for i in range(N):
        b.or_rht_encode_at(g[i], L, k, seed, base, enc[i])
    total = torch.empty(L, device=dev())
    count = torch.empty(L, dtype=torch.uint8, device=dev())
    b.or_masked_reduce(enc, m, N, L, total, count)
    mean = torch.where(count > 0, total / count.float().clamp(min=1), torch.zeros_like(total))
    out3 = torch.empty(L, device=dev())
    b.or_rht_decode_at(mean, L, k, seed, base, out3)
    outf = torch.empty(L, device=dev())
    countf = torch.empty(L, dtype=torch.uint8, device=dev())
    b.or_fused_path(g, m, N, L, k, seed, base, outf, countf)
    assert torch.equal(count, countf)
    want, want_count = orc.fused_path(to_np(g), to_np(m), k, seed, base)
    assert np.array_equal(to_np(count), want_count)
    assert rel_l2(to_np(out3), want) <= TOL["f32"] and rel_l2(to_np(outf), want) <= TOL["f32"]
    # about 1% of the entries of the other three workers are missing; the owner's are all there
    lost = 1.0 - to_np(count).astype(np.float64).mean() / N
    assert 0.004 < lost < 0.011 and to_np(count).min() >= 1


def test_no_drops_gives_exact_mean_of_integers(b):
    k, N = 12, 8
    L = 3 << k
    g = torch.randint(-4, 5, (N, L), device=dev(), generator=torch.Generator(device=dev()).manual_seed(3)).float()
    m = torch.full((N, L // 32), -1, dtype=torch.int32, device=dev())
    out = torch.empty(L, device=dev())
    count = torch.empty(L, dtype=torch.uint8, device=dev())
    b.or_fused_path(g, m, N, L, k, 9, 0, out, count)
    assert torch.equal(out, g.mean(dim=0)) and bool((count == N).all())


def test_tail_drop_is_dispersed(b, orc):
    # the paper's motivating pattern: the tail of one worker's shard never arrives
    from paper_2310_06993_amd import workloads as wl
    k, N = 10, 4
    L = 8 << k
    rng = np.random.default_rng(21)
    g = (rng.standard_normal((N, L)) * 1e-3).astype(np.float32)
    m = wl.tail_drop_masks(N, L, worker=2, fraction=0.1, device=dev())
    out = torch.empty(L, device=dev())
    count = torch.empty(L, dtype=torch.uint8, device=dev())
    b.or_fused_path(torch.from_numpy(g).to(dev()), m, N, L, k, 6, 0, out, count)
    want, want_count = orc.fused_path(g, to_np(m), k, 6, 0)
    assert np.array_equal(to_np(count), want_count) and rel_l2(to_np(out), want) <= TOL["f32"]
    assert int((to_np(count) == N - 1).sum()) == int(L * 0.1) // 32 * 32


# ------------------------------------------------------------------ edges
def test_empty_inputs_and_streams(b):
    z = torch.empty(0, device=dev())
    b.or_rht_encode(z, 0, 10, 1, z)
    b.or_rht_decode(z, 0, 10, 1, z)
    b.or_masked_reduce(z, torch.empty(0, dtype=torch.int32, device=dev()), 4, 0, z,
                       torch.empty(0, dtype=torch.uint8, device=dev()))
    b.or_fused_path(z, torch.empty(0, dtype=torch.int32, device=dev()), 4, 0, 10, 1, 0, z, None)
    # a caller stream other than the current one
    s = torch.cuda.Stream()
    n, k = 5000, 8
    x = torch.randn(n, device=dev())
    enc1 = torch.empty(b.or_padded_len(n, k), device=dev())
    enc2 = torch.empty_like(enc1)
    b.or_rht_encode(x, n, k, 3, enc1)
    torch.cuda.synchronize()
    b.or_rht_encode(x, n, k, 3, enc2, stream=s)
    s.synchronize()
    assert torch.equal(enc1, enc2)


def test_errors_leave_outputs_untouched(b):
    n, k = 4096, 12
    x = torch.randn(n, device=dev())
    out = torch.full((n,), 7.0, device=dev())
    with pytest.raises(b.OptiReduceError) as e:
        b.or_rht_encode(x, n, 3, 1, out)
    assert e.value.status == 2
    with pytest.raises(b.OptiReduceError) as e:
        b.or_rht_encode_at(x, n, k, 1, 100, out)
    assert e.value.status == 4
    with pytest.raises(b.OptiReduceError) as e:
        b.or_rht_encode(x[1:], n - 1, k, 1, out)      # misaligned input
    assert e.value.status == 5
    with pytest.raises(b.OptiReduceError) as e:
        b.or_rht_encode(x, n - 100, k, 1, x)          # in place needs whole blocks
    assert e.value.status == 4
    with pytest.raises(b.OptiReduceError) as e:
        b.or_fused_path(torch.zeros((2, 1 << 16), device=dev()), torch.zeros((2, 2048), dtype=torch.int32, device=dev()),
                        2, 1 << 16, 16, 1, 0, torch.zeros(1 << 16, device=dev()), None, None)
    assert e.value.status == 6
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


@pytest.mark.parametrize("k,kind,long", [(12, "f32", 0), (10, "bf16", 0), (16, "f32", 0), (12, "f32", 20), (11, "bf16", 14),
                                         (14, "f32", 0), (13, "bf16", 0), (15, "bf16", 0)])
def test_batched_buckets_equal_single_calls(b, orc, k, kind, long):
    # buckets of different lengths in one call (more than 64 of them for k = 12: several launches)
    B = 1 << k
    N = 4
    # long: launches of more than 768 tiles, which take the other form of the kernel
    lens = [B * (long + 1 + j % 3) for j in range(70)] if k == 12 or long else [2 * B, B, 0, 3 * B]
    dt = torch.float32 if kind == "f32" else torch.bfloat16
    gen = torch.Generator(device=dev()).manual_seed(k)
    items, singles = [], []
    nws = max(b.or_workspace_bytes(L, k) for L in lens)
    ws = torch.empty(nws, dtype=torch.uint8, device=dev()) if nws else None
    for j, L in enumerate(lens):
        g = (torch.randn((N, L), device=dev(), generator=gen) * 1e-3).to(dt)
        m = torch.randint(-2 ** 31, 2 ** 31 - 1, (N, L // 32), device=dev(), generator=gen, dtype=torch.int64).to(torch.int32)
        m |= torch.randint(-2 ** 31, 2 ** 31 - 1, (N, L // 32), device=dev(), generator=gen, dtype=torch.int64).to(torch.int32)
        if L:
            m[j % N] = -1
        out = torch.full((L,), float("nan"), device=dev()).to(dt)
        cnt = torch.zeros(L, dtype=torch.uint8, device=dev()) if j % 2 == 0 else None
        items.append((g, m, out, cnt, L, 100 + j, j * 4 * max(B, 128)))
        out1 = torch.empty(L, dtype=dt, device=dev())
        cnt1 = torch.empty(L, dtype=torch.uint8, device=dev())
        (b.or_fused_path if kind == "f32" else b.or_fused_path_bf16)(g, m, N, L, k, 100 + j, j * 4 * max(B, 128), out1, cnt1, ws)
        singles.append((out1, cnt1))
    arr = b.make_buckets(items)
    b.or_fused_path_batched(arr, len(items), N, k, kind == "bf16", ws)
    torch.cuda.synchronize()
    for (g, m, out, cnt, L, seed, base), (out1, cnt1) in zip(items, singles):
        assert torch.equal(out.view(torch.int16 if kind == "bf16" else torch.int32),
                           out1.view(torch.int16 if kind == "bf16" else torch.int32))
        if cnt is not None:
            assert torch.equal(cnt, cnt1)
    # and one of them against the oracle
    g, m, out, cnt, L, seed, base = items[1]
    want, _ = orc.fused_path(to_np(g), to_np(m), k, seed, base)
    assert rel_l2(to_np(out), want) <= TOL[kind]
    # a bad bucket anywhere in the list stops the whole call before anything runs
    bad = list(items)
    g, m, out, cnt, L, seed, base = bad[-1]
    bad[-1] = (g, m, out, cnt, L, seed, base + 32)
    items[0][2].fill_(5.0)
    with pytest.raises(b.OptiReduceError) as e:
        b.or_fused_path_batched(b.make_buckets(bad), len(bad), N, k, kind == "bf16", ws)
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert bool((items[0][2].float() == 5.0).all())


# ------------------------------------------------------------------ around the path
@pytest.mark.parametrize("N,L", [(4, 32 * 5), (8, 4096 * 3 + 64)])
def test_finalize_and_transform_off_path(b, orc, N, L):
    rng = np.random.default_rng(L)
    x = rng.standard_normal((N, L)).astype(np.float32)
    recv = rng.random((N, L)) > 0.3
    recv[:, 7] = False
    masks = pack_mask_np(recv)
    total = torch.empty(L, device=dev())
    count = torch.empty(L, dtype=torch.uint8, device=dev())
    b.or_masked_reduce(torch.from_numpy(x).to(dev()), masks_to_dev(masks), N, L, total, count)
    mean = torch.full((L,), float("nan"), device=dev())
    b.or_finalize(total, count, L, mean)
    ws, wc = orc.masked_reduce(x, masks)
    want = orc.finalize(ws, wc)
    assert rel_l2(to_np(mean), want) <= TOL["f32"] and float(mean[7]) == 0.0
    meanh = torch.zeros(L, dtype=torch.bfloat16, device=dev())
    b.or_finalize_bf16(total, count, L, meanh)
    assert rel_l2(to_np(meanh), want) <= TOL["bf16"]
    b.or_finalize(total, count, L, total)          # in place
    assert torch.equal(total, mean)
    # loss monitoring: exact
    tot = torch.full((1,), -1, dtype=torch.int64, device=dev())
    b.or_received_total(count, L, tot)
    assert int(tot.item()) == orc.received_total(wc) == int(recv.sum())


def test_received_total_large_and_empty(b):
    L = 32 * 100_003
    c = torch.randint(0, 256, (L,), dtype=torch.uint8, device=dev(), generator=torch.Generator(device=dev()).manual_seed(1))
    tot = torch.zeros(1, dtype=torch.int64, device=dev())
    b.or_received_total(c, L, tot)
    assert int(tot.item()) == int(c.to(torch.int64).sum().item())
    b.or_received_total(c, 0, tot)
    assert int(tot.item()) == 0


@pytest.mark.parametrize("k", [5, 10, 12, 14, 16])
def test_decode_masked(b, orc, k):
    B = 1 << k
    n = _sizes(k)[0]
    n_pad = b.or_padded_len(n, k)
    rng = np.random.default_rng(400 + k)
    agg = rng.standard_normal(n_pad).astype(np.float32)
    recv = rng.random(n_pad) > 0.05
    recv[64:128] = False
    mask = pack_mask_np(recv[None, :])[0]
    seed, base = 77, 2 * max(B, 128)
    poisoned = np.where(recv, agg, np.nan).astype(np.float32)     # lost entries are never read
    out = torch.empty(n, device=dev())
    b.or_rht_decode_masked(torch.from_numpy(poisoned).to(dev()), masks_to_dev(mask[None, :])[0], n, k, seed, base, out)
    assert rel_l2(to_np(out), orc.rht_decode_masked(agg, mask, n, k, seed, base)) <= TOL["f32"]
    outh = torch.empty(n, dtype=torch.bfloat16, device=dev())
    b.or_rht_decode_masked_bf16(torch.from_numpy(poisoned).to(dev()), masks_to_dev(mask[None, :])[0], n, k, seed, base, outh)
    assert rel_l2(to_np(outh), orc.rht_decode_masked(agg, mask, n, k, seed, base, out_dtype=np.uint16)) <= TOL["bf16"]
    full = torch.full((n_pad // 32,), -1, dtype=torch.int32, device=dev())
    out2 = torch.empty(n, device=dev())
    b.or_rht_decode_masked(torch.from_numpy(agg).to(dev()), full, n, k, seed, base, out2)
    out3 = torch.empty(n, device=dev())
    b.or_rht_decode_at(torch.from_numpy(agg).to(dev()), n, k, seed, base, out3)
    assert torch.equal(out2, out3)


@pytest.mark.parametrize("G,M,L", [(2, 2, 64), (4, 4, 32 * 300 + 32), (16, 3, 4096)])
def test_two_level_reduce(b, orc, G, M, L):
    rng = np.random.default_rng(G * 100 + M)
    x = rng.standard_normal((G * M, L)).astype(np.float32)
    recv = rng.random((G * M, L)) > 0.2
    masks = pack_mask_np(recv)
    sums = torch.empty((G, L), device=dev())
    counts = torch.empty((G, L), dtype=torch.uint8, device=dev())
    xd, md = torch.from_numpy(x).to(dev()), masks_to_dev(masks)
    for g in range(G):
        b.or_masked_reduce(xd[g * M:(g + 1) * M], md[g * M:(g + 1) * M], M, L, sums[g], counts[g])
    recv2 = rng.random((G, L)) > 0.15
    m2 = pack_mask_np(recv2)
    total = torch.empty(L, device=dev())
    count = torch.empty(L, dtype=torch.uint8, device=dev())
    sums_poisoned = torch.where(torch.from_numpy(recv2).to(dev()), sums, torch.full_like(sums, float("nan")))
    b.or_masked_reduce_pairs(sums_poisoned, counts, masks_to_dev(m2), G, L, total, count)
    ws, wc = orc.masked_reduce_pairs(to_np(sums), to_np(counts), m2)
    assert np.array_equal(to_np(count), wc) and rel_l2(to_np(total), ws) <= TOL["f32"]
    # the same as one level with a lost group = all its members lost (counts exactly, sums to rounding)
    w1, c1 = orc.masked_reduce(x, pack_mask_np(recv & np.repeat(recv2, M, axis=0)))
    assert np.array_equal(to_np(count), c1) and rel_l2(to_np(total), w1) <= TOL["f32"]


@pytest.mark.parametrize("k,kind", [(8, "f32"), (11, "f32"), (12, "f32"), (12, "bf16")])
def test_fused_forms_on_both_sides_of_the_grid_size_switch(b, orc, k, kind):
    """Launches of up to 768 tiles use the kernel form that prefetches the next worker's tile, larger ones
    the plain form: same arithmetic, so a shard of 769 tiles must reproduce, bit for bit, what its first 768
    tiles give as a shard of their own; sampled blocks of the large launch are checked against the oracle."""
    N = 3
    tile = max(1 << k, 1024)
    L_small, L_big = 768 * tile, 769 * tile
    g = torch.Generator(device=dev()).manual_seed(40 + k)
    raw = torch.randn((N, L_big), generator=g, device=dev()) * 1e-3
    recv = torch.rand((N, L_big), generator=g, device=dev()) > 0.02
    recv[0] = True
    words = recv.view(N, L_big // 32, 32).to(torch.int64)
    masks = (words << torch.arange(32, device=dev(), dtype=torch.int64)).sum(dim=2)
    masks = torch.where(masks >= 2 ** 31, masks - 2 ** 32, masks).to(torch.int32).contiguous()
    if kind == "bf16":
        raw = raw.to(torch.bfloat16)
    seed, base = 77 + k, 0
    fused = b.or_fused_path if kind == "f32" else b.or_fused_path_bf16
    out_big = torch.empty(L_big, dtype=raw.dtype, device=dev())
    cnt_big = torch.empty(L_big, dtype=torch.uint8, device=dev())
    fused(raw, masks, N, L_big, k, seed, base, out_big, cnt_big, _workspace(b, L_big, k))
    raw_s = raw[:, :L_small].contiguous()
    masks_s = masks[:, : L_small // 32].contiguous()
    out_s = torch.empty(L_small, dtype=raw.dtype, device=dev())
    cnt_s = torch.empty(L_small, dtype=torch.uint8, device=dev())
    fused(raw_s, masks_s, N, L_small, k, seed, base, out_s, cnt_s, _workspace(b, L_small, k))
    torch.cuda.synchronize()
    assert torch.equal(out_big[:L_small].view(torch.int32 if kind == "f32" else torch.int16),
                       out_s.view(torch.int32 if kind == "f32" else torch.int16))
    assert torch.equal(cnt_big[:L_small], cnt_s)
    # oracle on the first, a middle and the last tile of the large launch
    for t in (0, 400, 768):
        sl = slice(t * tile, (t + 1) * tile)
        r = to_np(raw[:, sl].contiguous())
        m = to_np(masks[:, t * tile // 32:(t + 1) * tile // 32].contiguous())
        want, want_count = orc.fused_path(r, m, k, seed, base + t * tile)
        assert np.array_equal(to_np(cnt_big[sl]), want_count)
        assert rel_l2(to_np(out_big[sl]), want) <= TOL[kind], (k, kind, t)


def test_seeded_sweep_of_shapes_through_every_route(b, orc):
    """Twenty seeded draws of (block size, workers, blocks, type, loss rate): the fused path, reduce+decode
    on the library's own encode output, and encode -> masked reduce -> finalize+decode must all land on the
    oracle, with identical counts."""
    rng = np.random.default_rng(20231006)
    for case in range(20):
        k = int(rng.integers(5, 17))
        N = int(rng.integers(1, 12))
        blocks = int(rng.integers(1, 5)) if k >= 13 else int(rng.integers(1, 40))
        kind = "f32" if rng.random() < 0.6 else "bf16"
        loss = float(rng.choice([0.0, 0.01, 0.2]))
        L = blocks << k
        raw32 = (rng.standard_normal((N, L)) * 1e-3).astype(np.float32)
        recv = rng.random((N, L)) >= loss
        recv[case % N] = True
        masks = pack_mask_np(recv)
        md = masks_to_dev(masks)
        seed, base = int(rng.integers(1, 2 ** 62)), int(rng.integers(0, 1000)) * max(1 << k, 128)
        tag = (case, k, N, blocks, kind, loss)
        ws = _workspace(b, L, k)
        cnt_f = torch.empty(L, dtype=torch.uint8, device=dev())
        cnt_r = torch.empty(L, dtype=torch.uint8, device=dev())
        cnt_3 = torch.empty(L, dtype=torch.uint8, device=dev())
        tot = torch.empty(L, device=dev())
        if kind == "f32":
            raw = raw32
            gd = torch.from_numpy(raw).to(dev())
            out_f, out_r, out_3 = (torch.empty(L, device=dev()) for _ in range(3))
            enc = torch.empty((N, L), device=dev())
            b.or_fused_path(gd, md, N, L, k, seed, base, out_f, cnt_f, ws)
            for i in range(N):
                b.or_rht_encode_at(gd[i], L, k, seed, base, enc[i])
            b.or_reduce_decode(enc, md, N, L, k, seed, base, out_r, cnt_r, ws)
            b.or_masked_reduce(enc, md, N, L, tot, cnt_3)
            b.or_finalize_decode(tot, cnt_3, L, k, seed, base, out_3)
        else:
            raw = _bf16_bits(raw32)
            gd = _dev_bf16(raw)
            out_f, out_r, out_3 = (torch.empty(L, dtype=torch.bfloat16, device=dev()) for _ in range(3))
            enc = torch.empty((N, L), dtype=torch.bfloat16, device=dev())
            b.or_fused_path_bf16(gd, md, N, L, k, seed, base, out_f, cnt_f, ws)
            for i in range(N):
                b.or_rht_encode_bf16(gd[i], L, k, seed, base, enc[i])
            b.or_reduce_decode_bf16(enc, md, N, L, k, seed, base, out_r, cnt_r, ws)
            b.or_masked_reduce_bf16(enc, md, N, L, tot, cnt_3)
            b.or_finalize_decode_bf16(tot, cnt_3, L, k, seed, base, out_3)
        want, want_count = orc.fused_path(raw, masks, k, seed, base)
        for name, out, cnt in (("fused", out_f, cnt_f), ("reduce_decode", out_r, cnt_r), ("three calls", out_3, cnt_3)):
            assert np.array_equal(to_np(cnt), want_count), (tag, name)
            assert rel_l2(to_np(out), want) <= TOL[kind], (tag, name)
