"""Several buckets per call (Sec. 3.1.1 footnote: DDP hands the collective 25 MB buckets): the batched forms of
the fused path and of the separate calls against single-bucket calls, the oracle and a popcount of the masks,
including the GPT-2-XL-sized configuration at its real shape (238 buckets, 16 workers), the launch shape that
bench.py times."""
import numpy as np
import pytest
import torch

from _util import TOL, dev, rel_l2, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def b():
    import paper_2310_06993_amd.binding as binding
    assert torch.cuda.is_available()
    return binding


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def _popcount_counts(m, L):
    """uint8 [L]: per entry, how many workers' bits are set (torch ops only)."""
    shifts = torch.arange(32, device=m.device, dtype=torch.int32)
    total = torch.zeros(L, dtype=torch.uint8, device=m.device)
    for i in range(m.shape[0]):
        total += ((m[i].unsqueeze(1) >> shifts) & 1).to(torch.uint8).reshape(-1)
    return total


def test_gpt2_xl_sized_batched_at_full_shape(b, orc):
    """Every bucket of the GPT-2-XL-sized gradient in one or_fused_path_batched call: 237 buckets of 6,553,600
    entries (shard 409,600 = 100 tiles) and the short last one (shard 278,528), 16 workers, block 2^12."""
    from paper_2310_06993_amd import workloads as wl
    cfg = wl.CONFIGS["gpt2_xl"]
    N, k, B = cfg.workers, cfg.block_log2, cfg.block
    buckets = cfg.buckets()
    assert len(buckets) == 238 and N == 16 and k == 12
    items = []
    for j, (first, n) in enumerate(buckets):
        shard = j % N
        L = cfg.shard_len(n)
        g = wl.make_grads(wl.scaled(cfg, n, seed=1000 + j), dev(), shard=shard)
        m = wl.make_masks(wl.scaled(cfg, n, seed=1000 + j), dev(), shard=shard)
        out = torch.full((L,), float("nan"), device=dev())
        cnt = torch.full((L,), 255, dtype=torch.uint8, device=dev())
        items.append((g, m, out, cnt, L, cfg.seed + j, shard * L))
    assert items[0][4] == 409_600 and items[-1][4] == 278_528
    totals = torch.full((len(items),), -1, dtype=torch.int64, device=dev())
    arr = b.make_buckets(items)
    b.or_fused_path_batched_monitored(arr, len(items), N, k, False, totals)
    torch.cuda.synchronize()
    # received counts of every bucket, every entry, against a popcount of the masks; and the loss statistic
    got_totals = totals.cpu().numpy()
    for j, (g, m, out, cnt, L, seed, base) in enumerate(items):
        want = _popcount_counts(m, L)
        assert torch.equal(cnt, want), j
        assert int(got_totals[j]) == int(want.sum(dtype=torch.int64)), j
        assert not bool(torch.isnan(out).any()), j
    # sampled blocks against the oracle: first bucket, both sides of every launch boundary, the short last one
    nl = -(-len(items) // 64)
    per = -(-len(items) // nl)
    picks = {0, 1, len(items) - 2, len(items) - 1}
    for l in range(1, nl):
        picks |= {l * per - 1, l * per}
    picks |= {63, 64, 127, 128, 191, 192}
    rng = np.random.default_rng(4)
    worst = 0.0
    for j in sorted(picks):
        g, m, out, cnt, L, seed, base = items[j]
        for blk in sorted({0, L // B - 1, int(rng.integers(0, L // B))}):
            gs = to_np(g[:, blk * B:(blk + 1) * B].contiguous())
            ms = to_np(m[:, blk * B // 32:(blk + 1) * B // 32].contiguous())
            want, wcnt = orc.fused_path(gs, ms, k, seed, base + blk * B)
            assert np.array_equal(to_np(cnt[blk * B:(blk + 1) * B]), wcnt), (j, blk)
            err = rel_l2(to_np(out[blk * B:(blk + 1) * B]), want)
            worst = max(worst, err)
            assert err <= TOL["f32"], (j, blk, err)
    # the same buckets one call each: identical bits
    for j in (0, 64, 237):
        g, m, out, cnt, L, seed, base = items[j]
        out1 = torch.empty_like(out)
        cnt1 = torch.empty_like(cnt)
        b.or_fused_path(g, m, N, L, k, seed, base, out1, cnt1)
        assert torch.equal(_bits(out), _bits(out1)) and torch.equal(cnt, cnt1)


def _random_buckets(N, lens, k, dt, seed):
    B = 1 << k
    gen = torch.Generator(device=dev()).manual_seed(seed)
    out = []
    for j, L in enumerate(lens):
        g = (torch.randn((N, L), device=dev(), generator=gen) * 1e-3).to(dt)
        m = torch.randint(-2 ** 31, 2 ** 31 - 1, (N, L // 32), device=dev(), generator=gen, dtype=torch.int64).to(torch.int32)
        m |= torch.randint(-2 ** 31, 2 ** 31 - 1, (N, L // 32), device=dev(), generator=gen, dtype=torch.int64).to(torch.int32)
        if L:
            m[j % N] = -1
        out.append((g, m, L, 300 + j, j * 4 * max(B, 128)))
    return out


@pytest.mark.parametrize("k,kind", [(12, "f32"), (12, "bf16"), (10, "f32"), (14, "bf16"), (13, "f32"), (16, "bf16")])
def test_empty_buckets_among_many_and_totals(b, orc, k, kind):
    """More than 64 buckets with empty ones scattered among them (also first and last), through the fused and
    the reduce+decode batched forms: equal to single calls bit for bit, untouched outputs nowhere, totals equal
    to the oracle's count of arrivals (0 for an empty bucket)."""
    B, N = 1 << k, 5
    dt = torch.float32 if kind == "f32" else torch.bfloat16
    nb = 150 if k <= 12 else 9
    lens = [0 if j % 7 in (0, 3) or j == nb - 1 else B * (1 + j % 3) for j in range(nb)]
    raw = _random_buckets(N, lens, k, dt, seed=k)
    nws = max(b.or_workspace_bytes(L, k) for L in lens)
    ws = torch.empty(nws, dtype=torch.uint8, device=dev()) if nws else None
    single = b.or_fused_path if kind == "f32" else b.or_fused_path_bf16
    enc_fn = b.or_rht_encode_at if kind == "f32" else b.or_rht_encode_bf16
    rdec = b.or_reduce_decode if kind == "f32" else b.or_reduce_decode_bf16
    fused_items, rd_items, refs = [], [], []
    for g, m, L, seed, base in raw:
        enc = torch.empty_like(g)
        for i in range(N):
            if L:
                enc_fn(g[i], L, k, seed, base, enc[i])
        o1, c1 = torch.empty(L, dtype=dt, device=dev()), torch.empty(L, dtype=torch.uint8, device=dev())
        o2, c2 = torch.empty(L, dtype=dt, device=dev()), torch.empty(L, dtype=torch.uint8, device=dev())
        single(g, m, N, L, k, seed, base, o1, c1, ws)
        rdec(enc, m, N, L, k, seed, base, o2, c2, ws)
        refs.append((o1, c1, o2, c2))
        fused_items.append((g, m, torch.full((L,), float("nan"), device=dev()).to(dt),
                            torch.full((L,), 255, dtype=torch.uint8, device=dev()), L, seed, base))
        rd_items.append((enc, m, torch.full((L,), float("nan"), device=dev()).to(dt),
                         torch.full((L,), 255, dtype=torch.uint8, device=dev()), L, seed, base))
    t1 = torch.full((nb,), -1, dtype=torch.int64, device=dev())
    t2 = torch.full((nb,), -1, dtype=torch.int64, device=dev())
    b.or_fused_path_batched_monitored(b.make_buckets(fused_items), nb, N, k, kind == "bf16", t1, ws)
    b.or_reduce_decode_batched(b.make_buckets(rd_items), nb, N, k, kind == "bf16", t2, ws)
    torch.cuda.synchronize()
    t1, t2 = t1.cpu().numpy(), t2.cpu().numpy()
    for j in range(nb):
        o1, c1, o2, c2 = refs[j]
        assert torch.equal(_bits(fused_items[j][2]), _bits(o1)) and torch.equal(fused_items[j][3], c1), j
        assert torch.equal(_bits(rd_items[j][2]), _bits(o2)) and torch.equal(rd_items[j][3], c2), j
        want_total = orc.received_total(to_np(c1))
        assert int(t1[j]) == want_total and int(t2[j]) == want_total, (j, t1[j], t2[j], want_total)
    assert int(t1[0]) == 0 and int(t1[nb - 1]) == 0
    # one non-empty bucket of each against the oracle
    j = 1
    g, m, L, seed, base = raw[j]
    want, wcnt = orc.fused_path(to_np(g), to_np(m), k, seed, base)
    assert rel_l2(to_np(fused_items[j][2]), want) <= TOL[kind]
    assert rel_l2(to_np(rd_items[j][2]), want) <= TOL[kind]
    assert np.array_equal(to_np(fused_items[j][3]), wcnt) and np.array_equal(to_np(rd_items[j][3]), wcnt)
    # totals == NULL is accepted
    b.or_reduce_decode_batched(b.make_buckets(rd_items), nb, N, k, kind == "bf16", None, ws)
    torch.cuda.synchronize()


@pytest.mark.parametrize("k,kind", [(12, "f32"), (12, "bf16"), (9, "f32"), (14, "f32"), (15, "bf16")])
def test_masked_reduce_and_finalize_decode_batched(b, orc, k, kind):
    """or_masked_reduce_batched and or_finalize_decode_batched on many buckets (some empty) equal the single
    calls bit for bit; one bucket of each against the oracle."""
    B, N = 1 << k, 6
    dt = torch.float32 if kind == "f32" else torch.bfloat16
    nb = 140 if k <= 12 else 7
    lens = [0 if j % 9 == 4 else B * (1 + j % 4) for j in range(nb)]
    raw = _random_buckets(N, lens, k, dt, seed=100 + k)
    red1 = b.or_masked_reduce if kind == "f32" else b.or_masked_reduce_bf16
    fdec1 = b.or_finalize_decode if kind == "f32" else b.or_finalize_decode_bf16
    items, refs = [], []
    for g, m, L, seed, base in raw:
        s1, c1 = torch.empty(L, device=dev()), torch.empty(L, dtype=torch.uint8, device=dev())
        o1 = torch.empty(L, dtype=dt, device=dev())
        red1(g, m, N, L, s1, c1)
        if L:
            fdec1(s1, c1, L, k, seed, base, o1)
        refs.append((s1, c1, o1))
        items.append((g, m, torch.full((L,), float("nan"), device=dev()),
                      torch.full((L,), 255, dtype=torch.uint8, device=dev()),
                      torch.full((L,), float("nan"), device=dev()).to(dt), L, seed, base))
    arr = b.make_stage_buckets(items)
    b.or_masked_reduce_batched(arr, nb, N, kind == "bf16")
    b.or_finalize_decode_batched(arr, nb, k, kind == "bf16")
    torch.cuda.synchronize()
    for j in range(nb):
        s1, c1, o1 = refs[j]
        assert torch.equal(items[j][2].view(torch.int32), s1.view(torch.int32)), j
        assert torch.equal(items[j][3], c1), j
        assert torch.equal(_bits(items[j][4]), _bits(o1)), j
    j = 2
    g, m, L, seed, base = raw[j]
    ws_, wc = orc.masked_reduce(to_np(g), to_np(m))
    assert np.array_equal(to_np(items[j][3]), wc) and rel_l2(to_np(items[j][2]), ws_) <= TOL["f32"]
    want = orc.rht_decode(orc.finalize(ws_, wc), L, k, seed, base, out_dtype=np.uint16 if kind == "bf16" else None)
    assert rel_l2(to_np(items[j][4]), want) <= TOL[kind]
    # a bad bucket anywhere stops the whole call before anything runs
    items[0][2].fill_(5.0)
    bad = list(items)
    sh, m, t, c, o, L, seed, base = bad[-1]
    bad[-1] = (sh, m, t, c, o, L + 16, seed, base)
    with pytest.raises(b.OptiReduceError) as e:
        b.or_masked_reduce_batched(b.make_stage_buckets(bad), nb, N, kind == "bf16")
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert bool((items[0][2] == 5.0).all())


def test_timing_events_span_every_launch_of_a_batched_call(b):
    """or_time_next_call on a call that enqueues several kernels: the start event rides on the first launch and
    the stop event on the last, so the elapsed time covers all of them (at least the sum of what the same
    launches take alone would be too strict a bound on a shared GPU: it must exceed the longest of them)."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]

    def events():
        a, z = ctypes.c_void_p(), ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(a)) == 0 and hip.hipEventCreate(ctypes.byref(z)) == 0
        return a, z

    def elapsed(a, z):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), a, z) == 0
        return ms.value

    k, N = 12, 8
    lens = [100 << k] * 130          # three launches
    raw = _random_buckets(N, lens, k, torch.float32, seed=9)
    items = [(g, m, torch.empty(L, device=dev()), None, L, seed, base) for g, m, L, seed, base in raw]
    arr = b.make_buckets(items)
    b.or_fused_path_batched(arr, len(items), N, k, False)
    torch.cuda.synchronize()
    a, z = events()
    b.or_time_next_call(a, z)
    b.or_fused_path_batched(arr, len(items), N, k, False)
    torch.cuda.synchronize()
    whole = elapsed(a, z)
    a1, z1 = events()
    b.or_time_next_call(a1, z1)
    b.or_fused_path_batched(b.make_buckets(items[:44]), 44, N, k, False)
    torch.cuda.synchronize()
    third = elapsed(a1, z1)
    assert whole > 1.6 * third > 0.0, (whole, third)      # three launches against one; the margin is for a noisy box
    for e in (a, z, a1, z1):
        hip.hipEventDestroy(e)
