"""Pins for the CPU oracle: every check compares the oracle with something other than itself
(published vectors, dense matrix products, closed forms, invariants, library routines)."""
import os

import numpy as np
import pytest
import scipy.linalg
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def dense_hadamard(B):
    """H[u][v] = (-1)^popcount(u & v), written out entry by entry."""
    u = np.arange(B)
    pc = np.zeros((B, B), np.int64)
    a = u[:, None] & u[None, :]
    while a.any():
        pc += a & 1
        a >>= 1
    return np.where(pc & 1, -1.0, 1.0)


def signs_pm1(orc, seed, first, count):
    return 1.0 - 2.0 * orc.sign_bits(seed, first, count).astype(np.float64)


def pack_mask(received):
    """bool [N, L] -> uint32 [N, L/32], entry 32w+j is bit j of word w."""
    r = np.asarray(received, bool)
    N, L = r.shape
    assert L % 32 == 0
    w = r.reshape(N, L // 32, 32).astype(np.uint64) << np.arange(32, dtype=np.uint64)
    return w.sum(axis=2).astype(np.uint32)


# ------------------------------------------------------------------ random diagonal
def test_philox_known_answers(orc):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        got = orc.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in got] == v[6:10]


def test_sign_stream_layout_and_balance(orc):
    seed = (0xDEADBEEF << 32) | 0x12345678
    # entry i takes bit (i mod 128), least significant first, of the output for counter i div 128,
    # key = (low half of seed, high half of seed)
    first = 5 * 128 + 17
    bits = orc.sign_bits(seed, first, 300)
    for j in (0, 1, 110, 111, 150, 299):
        i = first + j
        w = orc.philox4x32_10([i >> 7, 0, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        b = i & 127
        assert bits[j] == (int(w[b >> 5]) >> (b & 31)) & 1
    # counters above 2^32 use the second counter word
    i = (1 << 39) + 77
    w = orc.philox4x32_10([(i >> 7) & 0xFFFFFFFF, i >> 39, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
    assert orc.sign_bits(seed, i, 1)[0] == (int(w[(i & 127) >> 5]) >> (i & 31)) & 1
    # fair coin: within 5 sigma on a million draws, and seeds differ
    n = 1 << 20
    ones = int(orc.sign_bits(3, 0, n).sum())
    assert abs(ones - n / 2) < 5 * np.sqrt(n) / 2
    assert (orc.sign_bits(3, 0, 4096) != orc.sign_bits(4, 0, 4096)).mean() > 0.4


# ------------------------------------------------------------------ Hadamard
@pytest.mark.parametrize("k", range(0, 9))
def test_encode_equals_dense_matrix_product(orc, k):
    B = 1 << k
    H = dense_hadamard(B)
    rng = np.random.default_rng(100 + k)
    for seed, nblocks, tail in ((1, 1, 0), (7, 3, 0), (2**40 + 5, 2, max(1, B // 3) if B > 1 else 0)):
        n = nblocks * B - (B - tail if tail else 0)
        x = rng.standard_normal(n)
        base = 0
        got = orc.rht_encode(x, k, seed, base)
        n_pad = orc.padded_len(n, k)
        assert got.size == n_pad and n_pad % B == 0 and n_pad - n < B
        xp = np.zeros(n_pad)
        xp[:n] = x
        want = np.empty(n_pad)
        s = signs_pm1(orc, seed, base, n_pad)
        for b in range(n_pad // B):
            sl = slice(b * B, (b + 1) * B)
            want[sl] = H @ (s[sl] * xp[sl]) / np.sqrt(B)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12 * max(1.0, np.abs(want).max()))
        # decode is the inverse, also against the dense product
        dec = orc.rht_decode(got, n, k, seed, base)
        np.testing.assert_allclose(dec, x, rtol=0, atol=1e-12 * max(1.0, np.abs(x).max()))
        want_dec = np.empty(n_pad)
        y = rng.standard_normal(n_pad)
        for b in range(n_pad // B):
            sl = slice(b * B, (b + 1) * B)
            want_dec[sl] = s[sl] * (H @ y[sl]) / np.sqrt(B)
        np.testing.assert_allclose(orc.rht_decode(y, n, k, seed, base), want_dec[:n], rtol=0, atol=1e-12 * 20)


@pytest.mark.parametrize("k", [1, 4, 8, 10])
def test_hadamard_matches_scipy_sylvester(orc, k):
    B = 1 << k
    x = np.random.default_rng(k).standard_normal(B)
    np.testing.assert_allclose(orc.hadamard(x), scipy.linalg.hadamard(B).astype(np.float64) @ x,
                               rtol=0, atol=1e-10)


@pytest.mark.parametrize("k", [5, 10, 12, 16])
def test_hadamard_twice_is_B_times_identity_exactly(orc, k):
    B = 1 << k
    x = np.random.default_rng(k).integers(-50, 51, B).astype(np.float64)
    assert np.array_equal(orc.hadamard(orc.hadamard(x)), B * x)


def test_hadamard_of_unit_vectors(orc):
    # column v of H: entry u is (-1)^popcount(u&v); e_0 -> all ones, all ones -> B e_0
    B = 64
    assert np.array_equal(orc.hadamard(np.eye(B)[0]), np.ones(B))
    assert np.array_equal(orc.hadamard(np.ones(B)), B * np.eye(B)[0])
    e5 = orc.hadamard(np.eye(B)[5])
    assert np.array_equal(e5, dense_hadamard(B)[:, 5])
    # stride-1 pairs come first in natural order: e_1 -> +,-,+,-,...
    assert np.array_equal(orc.hadamard(np.eye(B)[1]), np.tile([1.0, -1.0], B // 2))


@pytest.mark.parametrize("k,dtype", [(10, np.float64), (12, np.float32), (7, np.float32), (11, np.float64)])
def test_parseval(orc, k, dtype):
    rng = np.random.default_rng(k)
    x = rng.standard_normal(5 * (1 << k) - 3).astype(dtype)
    y = orc.rht_encode(x, k, seed=9)
    nx, ny = np.linalg.norm(x.astype(np.float64)), np.linalg.norm(y.astype(np.float64))
    assert abs(nx - ny) / nx < (1e-12 if dtype == np.float64 else 1e-6)


# ------------------------------------------------------------------ aggregation
def _read_hand_example():
    d = {}
    for line in open(os.path.join(GOLDEN, "masked_sum_hand.txt")):
        if line[0] == "#":
            continue
        t = line.split()
        d[t[0]] = [float(v) for v in t[1:]]
    return d


def test_masked_sum_hand_example(orc):
    d = _read_hand_example()
    L = 32
    shards = np.zeros((3, L), np.float32)
    recv = np.zeros((3, L), bool)
    for i in range(3):
        shards[i, :4] = d["shard%d" % i]
        recv[i, [int(v) for v in d["recv%d" % i]]] = True
    total, count = orc.masked_reduce(shards, pack_mask(recv))
    assert total[:4].tolist() == d["sum"] and count[:4].tolist() == d["count"]
    assert not total[4:].any() and not count[4:].any()
    mean = orc.finalize(total, count)
    assert mean[:4].tolist() == d["mean"] and not mean[4:].any()


def test_mask_bit_order_and_worker_rows(orc):
    # entry 32w+j is bit j (LSB first) of word w of that worker's row
    N, L = 2, 96
    shards = np.arange(N * L, dtype=np.float32).reshape(N, L) + 1
    masks = np.zeros((N, L // 32), np.uint32)
    masks[0, 1] = 1 << 1       # worker 0, entry 33
    masks[1, 2] = 1 << 31      # worker 1, entry 95
    masks[1, 0] = 1            # worker 1, entry 0
    total, count = orc.masked_reduce(shards, masks)
    want = np.zeros(L, np.float32)
    want[33], want[95], want[0] = shards[0, 33], shards[1, 95], shards[1, 0]
    assert np.array_equal(total, want)
    assert count.sum() == 3 and count[33] == count[95] == count[0] == 1


def test_masked_reduce_matches_numpy_where(orc):
    rng = np.random.default_rng(5)
    N, L = 7, 32 * 9
    shards = rng.standard_normal((N, L)).astype(np.float32)
    recv = rng.random((N, L)) > 0.3
    total, count = orc.masked_reduce(shards, pack_mask(recv))
    want = np.where(recv, shards.astype(np.float64), 0.0).sum(axis=0)
    np.testing.assert_allclose(total, want, rtol=1e-6, atol=1e-6)
    assert np.array_equal(count, recv.sum(axis=0).astype(np.uint8))
    mean = orc.finalize(total, count)
    wm = np.divide(total.astype(np.float64), count, out=np.zeros(L), where=count > 0)
    np.testing.assert_allclose(mean, wm, rtol=1e-7)


def test_dropped_slots_are_never_read(orc):
    rng = np.random.default_rng(6)
    N, L = 5, 64
    shards = rng.standard_normal((N, L)).astype(np.float32)
    recv = rng.random((N, L)) > 0.4
    a = orc.masked_reduce(np.where(recv, shards, 0).astype(np.float32), pack_mask(recv))
    b = orc.masked_reduce(np.where(recv, shards, np.nan).astype(np.float32), pack_mask(recv))
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.isfinite(b[0]).all()


def test_all_dropped_gives_zero_mean(orc):
    shards = np.full((2, 32), 3.0, np.float32)
    total, count = orc.masked_reduce(shards, np.zeros((2, 1), np.uint32))
    assert not count.any() and not total.any() and not orc.finalize(total, count).any()


# ------------------------------------------------------------------ whole path
@pytest.mark.parametrize("k,N", [(10, 4), (6, 8), (12, 2)])
def test_no_drops_round_trip_is_exact_mean(orc, k, N):
    # integer data, power-of-two N, even k: every boundary value is exactly representable
    B = 1 << k
    L = 3 * B
    g = np.random.default_rng(k).integers(-8, 9, (N, L)).astype(np.float32)
    masks = np.full((N, L // 32), 0xFFFFFFFF, np.uint32)
    out, count = orc.fused_path(g, masks, k, seed=11, base_index=2 * B)
    assert np.array_equal(out, g.mean(axis=0).astype(np.float32))
    assert (count == N).all()
    # the same through the separate calls
    enc = np.stack([orc.rht_encode(g[i], k, 11, 2 * B) for i in range(N)])
    total, cnt = orc.masked_reduce(enc, masks)
    dec = orc.rht_decode(orc.finalize(total, cnt), L, k, 11, 2 * B)
    assert np.array_equal(dec, out)


def test_fused_is_the_composition_with_drops(orc):
    rng = np.random.default_rng(8)
    k, N = 8, 5
    L = 4 << k
    g = rng.standard_normal((N, L)).astype(np.float32)
    recv = rng.random((N, L)) > 0.1
    recv[2] = True
    masks = pack_mask(recv)
    out, count = orc.fused_path(g, masks, k, 3, 0)
    # definition written with the dense matrix, all in float64
    H = dense_hadamard(1 << k) / np.sqrt(1 << k)
    s = signs_pm1(orc, 3, 0, L)
    enc = np.stack([(H @ (s * g[i].astype(np.float64)).reshape(-1, 1 << k).T).T.reshape(-1) for i in range(N)])
    cnt = recv.sum(axis=0)
    mean = np.where(recv, enc, 0).sum(axis=0) / cnt
    want = s * (H @ mean.reshape(-1, 1 << k).T).T.reshape(-1)
    assert np.array_equal(count, cnt.astype(np.uint8))
    assert np.linalg.norm(out - want) / np.linalg.norm(want) < 1e-6


def test_one_lost_entry_is_spread_evenly(orc):
    # Sec. 3.3: a lost encoded entry perturbs every decoded entry of its block by the same
    # magnitude |y_j| / sqrt(B) and nothing outside the block; total squared error y_j^2.
    k = 8
    B = 1 << k
    x = np.random.default_rng(2).standard_normal(3 * B)
    y = orc.rht_encode(x, k, seed=5)
    j = B + 37
    y_lost = y.copy()
    y_lost[j] = 0.0
    err = orc.rht_decode(y_lost, x.size, k, 5) - x
    assert np.allclose(np.abs(err[B:2 * B]), abs(y[j]) / np.sqrt(B), rtol=1e-9)
    assert np.abs(err[:B]).max() < 1e-12 and np.abs(err[2 * B:]).max() < 1e-12
    assert np.isclose((err ** 2).sum(), y[j] ** 2, rtol=1e-9)
    # and without the transform the whole error lands on one entry
    assert np.isclose(np.abs(err).max() * np.sqrt(B), abs(y[j]), rtol=1e-9)


def test_tail_drop_error_is_dispersed(orc):
    # Sec. 3.3 / Sec. 1: with a tail drop the transformed bucket loses a little everywhere,
    # the plain bucket loses the tail entirely: the worst decoded entry is far better with HT.
    k, seed = 10, 4
    B = 1 << k
    x = np.random.default_rng(3).standard_normal(B)
    keep = np.arange(B) < int(0.9 * B)
    plain = np.where(keep, x, 0.0)
    enc = np.where(keep, orc.rht_encode(x, k, seed), 0.0)
    dec = orc.rht_decode(enc, B, k, seed)
    assert np.abs(dec - x).max() < 0.5 * np.abs(plain - x).max()
    # same total energy lost up to sampling: unbiased either way, only the spread differs
    assert 0.5 < ((dec - x) ** 2).sum() / ((plain - x) ** 2).sum() < 2.0


def test_linearity_and_slice_property(orc):
    k = 7
    B = 1 << k
    rng = np.random.default_rng(4)
    x, z = rng.standard_normal(6 * B), rng.standard_normal(6 * B)
    e = lambda v, base=0: orc.rht_encode(v, k, 21, base)
    np.testing.assert_allclose(e(2.5 * x - 0.75 * z), 2.5 * e(x) - 0.75 * e(z), atol=1e-12)
    # encoding a block-aligned slice with base_index = slice start gives that slice of the whole
    np.testing.assert_array_equal(e(x[2 * B:5 * B], 2 * B), e(x)[2 * B:5 * B])
    assert not np.array_equal(e(x[2 * B:5 * B], 0), e(x)[2 * B:5 * B])
    full = orc.rht_decode(e(x), x.size, k, 21)
    part = orc.rht_decode(e(x)[2 * B:5 * B], 3 * B, k, 21, 2 * B)
    np.testing.assert_array_equal(part, full[2 * B:5 * B])


def test_shared_seed_makes_reduction_commute(orc):
    # sum of encodings = encoding of the sum only because every worker uses the same diagonal
    k = 6
    rng = np.random.default_rng(12)
    g = rng.standard_normal((3, 4 << k))
    same = sum(orc.rht_encode(g[i], k, 17) for i in range(3))
    np.testing.assert_allclose(same, orc.rht_encode(g.sum(axis=0), k, 17), atol=1e-12)
    diff = sum(orc.rht_encode(g[i], k, 17 + i) for i in range(3))
    assert not np.allclose(orc.rht_decode(diff, g.shape[1], k, 17), g.sum(axis=0), atol=1e-3)


# ------------------------------------------------------------------ bf16 boundary
def test_bf16_rounding_matches_library_and_ties(orc):
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(2000).astype(np.float32) * 1e-3,
                        np.array([0.0, -0.0, 1.0, np.inf, -np.inf, 3.4e38, 1e-40], np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(orc.float_to_bf16(x), want)
    ties = np.array([0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF], np.uint32).view(np.float32)
    assert orc.float_to_bf16(ties).tolist() == [0x3F80, 0x3F82, 0x3F81, 0x3F80]
    nan = orc.float_to_bf16(np.array([np.nan], np.float32))[0]
    assert (nan & 0x7F80) == 0x7F80 and (nan & 0x7F) != 0
    assert np.array_equal(orc.bf16_to_float(want[:100]),
                          torch.from_numpy(x[:100]).to(torch.bfloat16).float().numpy())


def test_bf16_path_rounds_only_at_boundaries(orc):
    k, N = 8, 4
    L = 2 << k
    rng = np.random.default_rng(9)
    g32 = (rng.standard_normal((N, L)) * 1e-3).astype(np.float32)
    g = orc.float_to_bf16(g32)
    recv = rng.random((N, L)) > 0.05
    recv[1] = True
    masks = pack_mask(recv)
    out, count = orc.fused_path(g, masks, k, 2, 0)
    gf = orc.bf16_to_float(g).astype(np.float64)
    H = dense_hadamard(1 << k) / np.sqrt(1 << k)
    s = signs_pm1(orc, 2, 0, L)
    enc = np.stack([(H @ (s * gf[i]).reshape(-1, 1 << k).T).T.reshape(-1) for i in range(N)])
    encw = torch.from_numpy(enc.astype(np.float32)).to(torch.bfloat16).double().numpy()
    np.testing.assert_array_equal(orc.bf16_to_float(orc.rht_encode(g[0], k, 2)).astype(np.float64), encw[0])
    mean = np.where(recv, encw, 0).sum(axis=0) / recv.sum(axis=0)
    want = s * (H @ mean.reshape(-1, 1 << k).T).T.reshape(-1)
    got = orc.bf16_to_float(out).astype(np.float64)
    assert np.linalg.norm(got - want) / np.linalg.norm(want) < 4e-3   # one bf16 rounding of the output
    assert np.array_equal(count, recv.sum(axis=0).astype(np.uint8))


# ------------------------------------------------------------------ second-stage loss, monitoring, two levels
def test_decode_masked_is_decode_of_zero_filled(orc):
    k, seed = 8, 13
    B = 1 << k
    n = 3 * B - 7
    rng = np.random.default_rng(31)
    agg = rng.standard_normal(orc.padded_len(n, k)).astype(np.float32)
    recv = rng.random(agg.size) > 0.05
    got = orc.rht_decode_masked(agg, pack_mask(recv[None, :])[0], n, k, seed, 2 * B)
    H = dense_hadamard(B) / np.sqrt(B)
    s = signs_pm1(orc, seed, 2 * B, agg.size)
    want = s * (H @ np.where(recv, agg.astype(np.float64), 0.0).reshape(-1, B).T).T.reshape(-1)
    np.testing.assert_allclose(got, want[:n], rtol=0, atol=2e-6)
    # all arrived: the plain decode, bit for bit
    full = np.full(agg.size // 32, 0xFFFFFFFF, np.uint32)
    assert np.array_equal(orc.rht_decode_masked(agg, full, n, k, seed, 2 * B), orc.rht_decode(agg, n, k, seed, 2 * B))
    # one aggregated entry lost in the broadcast: same magnitude |a_j|/sqrt(B) everywhere in its block
    one = full.copy()
    j = B + 5
    one[j // 32] &= ~np.uint32(1 << (j % 32))
    err = orc.rht_decode_masked(agg, one, agg.size, k, seed, 0).astype(np.float64) - \
        orc.rht_decode(agg, agg.size, k, seed, 0).astype(np.float64)
    assert np.allclose(np.abs(err[B:2 * B]), abs(agg[j]) / np.sqrt(B), rtol=1e-4)
    assert not err[:B].any() and not err[2 * B:].any()


def _bf16_bits_of(x64):
    """fp64 -> fp32 -> bf16 bit patterns through torch's conversions (round to nearest even both times)."""
    return torch.from_numpy(np.asarray(x64, np.float64).astype(np.float32)).to(torch.bfloat16).view(torch.int16) \
        .numpy().view(np.uint16)


def _equal_up_to_straddles(got, want):
    """bf16 bit patterns equal, except where the fp64 value sits within rounding noise of a rounding
    boundary (the butterfly and the dense product order their fp64 additions differently): at most one
    entry in 10^4 may differ, and then by one unit in the last place."""
    got, want = np.asarray(got, np.uint16), np.asarray(want, np.uint16)
    bad = np.flatnonzero(got != want)
    assert bad.size <= max(1, got.size // 10000), "%d of %d bf16 values differ" % (bad.size, got.size)
    for j in bad:
        assert abs(int(got[j]) - int(want[j])) == 1


@pytest.mark.parametrize("k", [5, 8])
def test_decode_to_bf16_is_the_dense_product_rounded_once(orc, k):
    # Sec. 3.3 / Sec. 4 decode with a bf16 result: g = D B^(-1/2) H m written out with the dense matrix in
    # fp64, then rounded to the output type (reading R7: bf16 only at the memory boundary)
    seed, B = 21, 1 << k
    base = 4 * max(B, 128)
    n = 3 * B - 5
    rng = np.random.default_rng(40 + k)
    agg = (rng.standard_normal(orc.padded_len(n, k)) * 1e-3).astype(np.float32)
    H = dense_hadamard(B) / np.sqrt(B)
    s = signs_pm1(orc, seed, base, agg.size)
    want = s * (H @ agg.astype(np.float64).reshape(-1, B).T).T.reshape(-1)
    got = orc.rht_decode(agg, n, k, seed, base, out_dtype=np.uint16)
    assert got.dtype == np.uint16 and got.shape == (n,)
    _equal_up_to_straddles(got, _bf16_bits_of(want[:n]))
    # a transposed operand, a dropped sign or a missing scale would be far outside one unit in the last place
    wrong = s * (agg.astype(np.float64).reshape(-1, B) @ H.T).reshape(-1) * np.sqrt(B)
    assert np.count_nonzero(got != _bf16_bits_of(wrong[:n])) > n // 2


@pytest.mark.parametrize("k", [5, 8])
def test_decode_masked_to_bf16_is_the_dense_product_of_the_zero_filled_mean(orc, k):
    # second-stage loss (Sec. 3.1.1 broadcast stage; reading R15) with a bf16 result
    seed, B = 22, 1 << k
    base = 2 * max(B, 128)
    n = 4 * B - 9
    rng = np.random.default_rng(50 + k)
    agg = (rng.standard_normal(orc.padded_len(n, k)) * 1e-3).astype(np.float32)
    recv = rng.random(agg.size) > 0.07
    poisoned = np.where(recv, agg, np.float32(np.nan))          # a lost slot is never read
    H = dense_hadamard(B) / np.sqrt(B)
    s = signs_pm1(orc, seed, base, agg.size)
    want = s * (H @ np.where(recv, agg.astype(np.float64), 0.0).reshape(-1, B).T).T.reshape(-1)
    got = orc.rht_decode_masked(poisoned, pack_mask(recv[None, :])[0], n, k, seed, base, out_dtype=np.uint16)
    assert got.dtype == np.uint16 and got.shape == (n,)
    _equal_up_to_straddles(got, _bf16_bits_of(want[:n]))
    # all arrived: the plain bf16 decode, bit for bit; and it differs from the masked result where loss hit
    full = np.full(agg.size // 32, 0xFFFFFFFF, np.uint32)
    plain = orc.rht_decode(agg, n, k, seed, base, out_dtype=np.uint16)
    assert np.array_equal(orc.rht_decode_masked(agg, full, n, k, seed, base, out_dtype=np.uint16), plain)
    assert np.count_nonzero(plain != got) > n // 4


def test_received_total_and_loss_fraction(orc):
    rng = np.random.default_rng(32)
    N, L = 6, 32 * 50
    recv = rng.random((N, L)) > 0.1
    _, count = orc.masked_reduce(rng.standard_normal((N, L)).astype(np.float32), pack_mask(recv))
    assert orc.received_total(count) == int(recv.sum())
    assert orc.received_total(np.full(1000, 255, np.uint8)) == 255000
    assert orc.received_total(np.zeros(0, np.uint8)) == 0


def test_two_level_reduce_equals_one_level(orc):
    # Sec. 3.1.2: aggregate inside each group, then across groups.  With every group aggregate
    # delivered this is the one-level aggregation (sums exactly representable here); a group aggregate
    # lost at the second level is the same as all of that group's members lost at that entry.
    rng = np.random.default_rng(33)
    G, M, L = 4, 3, 32 * 20
    x = rng.integers(-8, 9, (G * M, L)).astype(np.float32)
    recv = rng.random((G * M, L)) > 0.2
    masks = pack_mask(recv)
    sums = np.empty((G, L), np.float32)
    counts = np.empty((G, L), np.uint8)
    for g in range(G):
        sums[g], counts[g] = orc.masked_reduce(x[g * M:(g + 1) * M], masks[g * M:(g + 1) * M])
    all_ones = np.full((G, L // 32), 0xFFFFFFFF, np.uint32)
    t2, c2 = orc.masked_reduce_pairs(sums, counts, all_ones)
    t1, c1 = orc.masked_reduce(x, masks)
    assert np.array_equal(t2, t1) and np.array_equal(c2, c1)
    recv2 = rng.random((G, L)) > 0.25
    t2, c2 = orc.masked_reduce_pairs(sums, counts, pack_mask(recv2))
    t1, c1 = orc.masked_reduce(x, pack_mask(recv & np.repeat(recv2, M, axis=0)))
    assert np.array_equal(t2, t1) and np.array_equal(c2, c1)
    # hand-sized case: two groups, sums (3, 10) and counts (2, 1); only the second arrives at entry 0
    s = np.zeros((2, 32), np.float32); c = np.zeros((2, 32), np.uint8)
    s[:, 0] = [3, 10]; c[:, 0] = [2, 1]
    m = np.zeros((2, 1), np.uint32); m[1, 0] = 1
    t, cc = orc.masked_reduce_pairs(s, c, m)
    assert t[0] == 10 and cc[0] == 1 and not t[1:].any() and not cc[1:].any()


def test_loss_decision_hand_cases(orc):
    # Sec. 3.4 / Sec. 3.2.1 by hand: 8 workers x 1000 entries = 8000 sent
    # 7900 arrived -> loss 1.25 %: below the 2 % switch, below a 5 % skip threshold
    assert orc.loss_decision(7900, 8, 1000, 0.02, 0.05, 0.5, False) == (0, False, 0.0125)
    # 7800 arrived -> 2.5 %: transform goes on, update still applied
    assert orc.loss_decision(7800, 8, 1000, 0.02, 0.05, 0.5, False) == (0, True, 0.025)
    # exactly 2 % is not "exceeds"
    assert orc.loss_decision(7840, 8, 1000, 0.02, 0.05, 0.5, False)[:2] == (0, False)
    # once on, the transform stays on even with no loss at all
    assert orc.loss_decision(8000, 8, 1000, 0.02, 0.05, 0.5, True) == (0, True, 0.0)
    # 7000 arrived -> 12.5 %: skip; 3000 arrived -> 62.5 %: halt
    assert orc.loss_decision(7000, 8, 1000, 0.02, 0.05, 0.5, False) == (1, True, 0.125)
    assert orc.loss_decision(3000, 8, 1000, 0.02, 0.05, 0.5, False) == (2, True, 0.625)
    # a threshold above 1 switches that action off
    assert orc.loss_decision(0, 8, 1000, 0.02, 2.0, 2.0, False) == (0, True, 1.0)
