"""Seeded synthetic inputs shaped like the paper's workloads.  Shared by the tests and the benchmark.

This module only makes INPUTS (gradient slices and drop masks); none of the method's arithmetic
lives here and it imports neither the HIP binding nor the oracle.  Everything is torch, runs on
CPU or GPU, and is a pure function of (config, seed) on a given device type.

The five configurations stand in for the models the paper trains (its gradients, datasets and
checkpoints are not needed for this path): sizes are the parameter counts of ResNet-50,
BERT-large, GPT-2-XL and an 8B Llama; values are Gaussian with the stated extras; drops follow the
loss patterns the paper discusses (random loss, packet-sized runs, bursts, tail drops).

One node's view is simulated: the node owns shard `r` of the padded gradient and holds the r-th
slice of every worker.  Its own slice never crosses the network, so its mask row is all ones.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch


@dataclass(frozen=True)
class Config:
    name: str
    workers: int            # N
    dtype: str              # "f32" or "bf16"
    entries: int            # P, entries of one worker's gradient
    block_log2: int         # k
    sigma: float
    values: str             # "normal" | "outliers" | "layers"
    drops: str              # "iid_entry" | "iid_packet" | "gilbert"
    loss: float
    packet: int = 256       # entries per packet
    burst: float = 1.0      # mean burst length in packets (gilbert)
    bucket_entries: int = 0  # >0: the gradient is cut into buckets of this many entries (25 MiB fp32)
    seed: int = 1

    @property
    def block(self) -> int:
        return 1 << self.block_log2

    def padded_entries(self, entries: int | None = None) -> int:
        """P rounded up to a multiple of N*B so that every shard holds whole blocks."""
        q = self.workers * self.block
        p = self.entries if entries is None else entries
        return (p + q - 1) // q * q

    def shard_len(self, entries: int | None = None) -> int:
        return self.padded_entries(entries) // self.workers

    def buckets(self):
        """[(first entry, entries)] of the buckets of one gradient (a single bucket if unbucketed)."""
        if not self.bucket_entries:
            return [(0, self.entries)]
        out, pos = [], 0
        while pos < self.entries:
            n = min(self.bucket_entries, self.entries - pos)
            out.append((pos, n))
            pos += n
        return out


CONFIGS = {
    "tiny": Config("tiny", 4, "f32", 65_536, 10, 1e-3, "normal", "iid_entry", 0.01, seed=1),
    "resnet50": Config("resnet50", 8, "f32", 25_557_032, 12, 1e-3, "outliers", "iid_packet", 0.01, 256, seed=2),
    "bert_large": Config("bert_large", 8, "f32", 335_141_888, 14, 1.0, "layers", "gilbert", 0.02, 256, 8.0, seed=3),
    "gpt2_xl": Config("gpt2_xl", 16, "f32", 1_557_611_200, 12, 1e-3, "normal", "iid_packet", 0.05, 256,
                      bucket_entries=6_553_600, seed=4),
    "llama_8b": Config("llama_8b", 8, "bf16", 8_030_261_248, 16, 1e-4, "normal", "gilbert", 0.01, 512, 32.0, seed=5),
}
ORDER = ["tiny", "resnet50", "bert_large", "gpt2_xl", "llama_8b"]


def scaled(cfg: Config, entries: int, **kw) -> Config:
    """The same recipe on a smaller gradient (parity tests at sizes the oracle finishes in seconds)."""
    d = dict(cfg.__dict__)
    d.update(entries=entries, **kw)
    return Config(**d)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


_LAYER = 1 << 20  # "layers" recipe: consecutive segments of 2^20 entries share a scale


def make_grads(cfg: Config, device="cpu", shard: int = 0, entries: int | None = None, first: int = 0,
               chunk: int = 1 << 26) -> torch.Tensor:
    """Raw slices [N, L] of shard `shard` of every worker's gradient (float32 or bfloat16).

    `entries`/`first` select a bucket: the gradient cfg is asked about has `entries` entries and
    starts at global entry `first` (only the "layers" recipe looks at `first`).  Entries of the
    pad (global index >= entries) are zero.
    """
    n_total = cfg.entries if entries is None else entries
    N, L = cfg.workers, cfg.shard_len(n_total)
    dt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    out = torch.empty((N, L), dtype=dt, device=device)
    g = _gen(device, cfg.seed * 1_000_003 + shard * 7919 + 11)
    lo = shard * L
    for i in range(N):
        for c0 in range(0, L, chunk):
            c1 = min(L, c0 + chunk)
            x = torch.randn(c1 - c0, generator=g, device=device, dtype=torch.float32)
            if cfg.values == "outliers":
                big = torch.rand(c1 - c0, generator=g, device=device) < 0.01
                x = torch.where(big, x * 100.0, x)
            if cfg.values == "layers":
                idx = torch.arange(first + lo + c0, first + lo + c1, device=device) // _LAYER
                # log-uniform in [1e-5, 1e-2], a fixed function of the layer number and the seed
                u = ((idx * 2654435761 + cfg.seed * 97) % 1000003).to(torch.float32) / 1000003.0
                x = x * torch.pow(10.0, -5.0 + 3.0 * u)
            else:
                x = x * cfg.sigma
            valid = n_total - (lo + c0)
            if valid < c1 - c0:
                x[max(valid, 0):] = 0.0
            out[i, c0:c1] = x.to(dt)
    return out


def _pack_bits(received: torch.Tensor) -> torch.Tensor:
    """bool [N, L] -> int32 [N, L/32] bit patterns; entry 32w+j is bit j of word w."""
    N, L = received.shape
    w = received.view(N, L // 32, 32).to(torch.int64) << torch.arange(32, device=received.device)
    w = w.sum(dim=2)
    return torch.where(w >= 2 ** 31, w - 2 ** 32, w).to(torch.int32)


def _packets_to_words(ok: torch.Tensor, packet: int, L: int) -> torch.Tensor:
    """bool [N, packets] -> int32 words [N, L/32]: a packet covers `packet` consecutive entries."""
    assert packet % 32 == 0
    w = torch.where(ok, torch.tensor(-1, dtype=torch.int32, device=ok.device),
                    torch.tensor(0, dtype=torch.int32, device=ok.device))
    w = w.repeat_interleave(packet // 32, dim=1)
    return w[:, : L // 32].contiguous()


def _gilbert_packets(npk: int, loss: float, burst: float, g: torch.Generator, device) -> torch.Tensor:
    """Two-state burst-loss chain over packets (lost exactly in the Bad state).  Mean Bad run =
    `burst` packets, stationary loss = `loss`.  Built from alternating geometric run lengths."""
    r = 1.0 / burst                     # P(Bad -> Good)
    p = loss * r / (1.0 - loss)         # P(Good -> Bad)
    mean_cycle = 1.0 / p + 1.0 / r
    runs = int(npk / mean_cycle * 1.5) + 64
    while True:
        good = torch.empty(runs, device=device).geometric_(p, generator=g)
        bad = torch.empty(runs, device=device).geometric_(r, generator=g)
        start_bad = bool(torch.rand(1, generator=g, device=device).item() < loss)
        pair = torch.stack([bad, good] if start_bad else [good, bad], dim=1).reshape(-1).to(torch.int64)
        ends = torch.cumsum(pair, 0)
        if int(ends[-1]) >= npk:
            break
        runs *= 2
    run_of = torch.searchsorted(ends, torch.arange(npk, device=device), right=True)
    is_bad = (run_of % 2 == 0) if start_bad else (run_of % 2 == 1)
    return ~is_bad


def make_masks(cfg: Config, device="cpu", shard: int = 0, entries: int | None = None, self_worker: int | None = None,
               salt: int = 0) -> torch.Tensor:
    """Received-bit masks [N, L/32] (int32 bit patterns, 1 = arrived) for shard `shard`."""
    N, L = cfg.workers, cfg.shard_len(entries)
    g = _gen(device, cfg.seed * 2_000_003 + shard * 104729 + 13 + salt)
    me = shard % N if self_worker is None else self_worker
    if cfg.drops == "iid_entry":
        rows = []
        for i in range(N):
            rows.append(torch.rand(L, generator=g, device=device) >= cfg.loss)
        m = _pack_bits(torch.stack(rows))
    else:
        npk = (L + cfg.packet - 1) // cfg.packet
        if cfg.drops == "iid_packet":
            ok = torch.rand((N, npk), generator=g, device=device) >= cfg.loss
        elif cfg.drops == "gilbert":
            ok = torch.stack([_gilbert_packets(npk, cfg.loss, cfg.burst, g, device) for _ in range(N)])
        else:
            raise ValueError(cfg.drops)
        m = _packets_to_words(ok, cfg.packet, L)
    m[me] = -1
    return m


def tail_drop_masks(N: int, L: int, worker: int, fraction: float, device="cpu") -> torch.Tensor:
    """Everything arrives except the last `fraction` of one worker's shard (the paper's tail drop)."""
    m = torch.full((N, L // 32), -1, dtype=torch.int32, device=device)
    lost_words = int(L * fraction) // 32
    if lost_words:
        m[worker, L // 32 - lost_words:] = 0
    return m


def bytes_fused(N: int, L: int, elem_bytes: int, with_counts: bool = True) -> int:
    """Bytes the fused path must move: N raw slices and N mask rows in, one decoded shard (and the
    counts) out."""
    return N * L * elem_bytes + N * L // 8 + L * elem_bytes + (L if with_counts else 0)
