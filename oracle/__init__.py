"""CPU oracle for the OptiReduce gradient-bucket path.  TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front for ``optireduce_oracle.cpp`` (single-threaded C++,
double-precision interior arithmetic).  Only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; the product path never
does.  Nothing here imports the HIP binding.

Each function names the passage of the paper (arXiv 2310.06993) it follows; the
readings taken where the paper is silent are listed at the top of the C++ file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "optireduce_oracle.cpp")
_LIB = os.path.join(_HERE, "liboptireduce_oracle.so")

_u64, _int = C.c_uint64, C.c_int
_p = C.c_void_p


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (no HIP, no SIMD flags, -O2)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["g++", "-std=c++17", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fPIC", "-shared",
             _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.orc_padded_len.restype = _u64
        L.orc_padded_len.argtypes = [_u64, _int]
        L.orc_float_to_bf16.restype = C.c_uint16
        L.orc_float_to_bf16.argtypes = [C.c_float]
        L.orc_bf16_to_float.restype = C.c_float
        L.orc_bf16_to_float.argtypes = [C.c_uint16]
        L.orc_philox4x32_10.argtypes = [_p, _p, _p]
        L.orc_sign_bits.argtypes = [_u64, _u64, _u64, _p]
        L.orc_hadamard_f64.argtypes = [_p, _u64]
        for name in ("orc_rht_encode_f64", "orc_rht_encode_f32", "orc_rht_encode_bf16",
                     "orc_rht_decode_f64", "orc_rht_decode_f32", "orc_rht_decode_bf16"):
            getattr(L, name).argtypes = [_p, _u64, _int, _u64, _u64, _p]
        for name in ("orc_masked_reduce_f32", "orc_masked_reduce_bf16"):
            getattr(L, name).argtypes = [_p, _p, _int, _u64, _p, _p]
        L.orc_finalize.argtypes = [_p, _p, _u64, _p]
        for name in ("orc_rht_decode_masked_f32", "orc_rht_decode_masked_bf16"):
            getattr(L, name).argtypes = [_p, _p, _u64, _int, _u64, _u64, _p]
        L.orc_received_total.restype = _u64
        L.orc_received_total.argtypes = [_p, _u64]
        L.orc_masked_reduce_pairs.argtypes = [_p, _p, _p, _int, _u64, _p, _p]
        for name in ("orc_fused_path_f32", "orc_fused_path_bf16"):
            getattr(L, name).argtypes = [_p, _p, _int, _u64, _int, _u64, _u64, _p, _p]
        _lib = L
    return _lib


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a):
    return a.ctypes.data_as(_p)


# ----------------------------------------------------------------------------- pieces
def philox4x32_10(counter, key) -> np.ndarray:
    """Philox4x32-10 of Salmon et al. (SC'11): 4 counter words, 2 key words -> 4 words."""
    c = _arr(counter, np.uint32)
    k = _arr(key, np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, np.uint32)
    _load().orc_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def sign_bits(seed: int, first: int, count: int) -> np.ndarray:
    """1 where the shared random diagonal of Sec. 3.3 is -1, for entries first..first+count-1."""
    out = np.empty(count, np.uint8)
    _load().orc_sign_bits(seed, first, count, _ptr(out))
    return out


def padded_len(n: int, block_log2: int) -> int:
    return int(_load().orc_padded_len(n, block_log2))


def hadamard(x) -> np.ndarray:
    """Unnormalised natural-order Walsh-Hadamard transform of a power-of-two length vector (fp64)."""
    y = _arr(x, np.float64).copy()
    assert y.ndim == 1 and y.size & (y.size - 1) == 0 and y.size > 0
    _load().orc_hadamard_f64(_ptr(y), y.size)
    return y


def float_to_bf16(x) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even."""
    x = _arr(x, np.float32)
    L = _load()
    return np.array([L.orc_float_to_bf16(float(v)) for v in x.ravel()], np.uint16).reshape(x.shape)


def bf16_to_float(h) -> np.ndarray:
    h = _arr(h, np.uint16)
    return (h.astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------- the path
_ENC = {np.dtype(np.float64): ("orc_rht_encode_f64", np.float64),
        np.dtype(np.float32): ("orc_rht_encode_f32", np.float32),
        np.dtype(np.uint16): ("orc_rht_encode_bf16", np.uint16)}


def rht_encode(grad, block_log2: int, seed: int, base_index: int = 0) -> np.ndarray:
    """Sec. 3.3 encode of one bucket: shared random signs, blockwise Hadamard, B^(-1/2).

    dtype float64 -> unrounded result; float32 -> fp32 wire; uint16 -> bf16 in and bf16 wire.
    Returns padded_len(n) entries.
    """
    g = np.ascontiguousarray(grad)
    name, dt = _ENC[g.dtype]
    out = np.empty(padded_len(g.size, block_log2), dt)
    getattr(_load(), name)(_ptr(g), g.size, block_log2, seed, base_index, _ptr(out))
    return out


def masked_reduce(shards, masks):
    """Sec. 3.1.1 aggregation at the shard's owner over the entries that arrived.

    shards: [N, L] float32 or uint16 (bf16 bits); masks: [N, L/32] uint32, bit j of word w is
    entry 32w+j, 1 = arrived.  Returns (sum fp32 [L], count uint8 [L]).
    """
    s = np.ascontiguousarray(shards)
    m = _arr(masks, np.uint32)
    N, Ln = s.shape
    assert Ln % 32 == 0 and m.shape == (N, Ln // 32)
    total = np.empty(Ln, np.float32)
    count = np.empty(Ln, np.uint8)
    fn = "orc_masked_reduce_f32" if s.dtype == np.float32 else "orc_masked_reduce_bf16"
    assert s.dtype in (np.float32, np.uint16)
    getattr(_load(), fn)(_ptr(s), _ptr(m), N, Ln, _ptr(total), _ptr(count))
    return total, count


def finalize(total, count) -> np.ndarray:
    """The "averages" of Sec. 3.1.1 over what arrived: sum / count, 0 where count is 0."""
    t = _arr(total, np.float32)
    c = _arr(count, np.uint8)
    out = np.empty(t.size, np.float32)
    _load().orc_finalize(_ptr(t), _ptr(c), t.size, _ptr(out))
    return out


def rht_decode(agg, n: int, block_log2: int, seed: int, base_index: int = 0, out_dtype=None) -> np.ndarray:
    """Sec. 3.3 / Sec. 4 decode of the aggregated bucket; keeps the first n entries.

    agg float64 -> unrounded; agg float32 -> fp32 out, or bf16 bits with out_dtype=np.uint16.
    """
    a = np.ascontiguousarray(agg)
    assert a.size == padded_len(n, block_log2)
    if a.dtype == np.float64:
        out = np.empty(n, np.float64)
        fn = "orc_rht_decode_f64"
    elif out_dtype is not None and np.dtype(out_dtype) == np.uint16:
        a = _arr(a, np.float32)
        out = np.empty(n, np.uint16)
        fn = "orc_rht_decode_bf16"
    else:
        a = _arr(a, np.float32)
        out = np.empty(n, np.float32)
        fn = "orc_rht_decode_f32"
    getattr(_load(), fn)(_ptr(a), n, block_log2, seed, base_index, _ptr(out))
    return out


def rht_decode_masked(agg, mask, n: int, block_log2: int, seed: int, base_index: int = 0, out_dtype=None):
    """Decode after second-stage loss (Sec. 3.1.1 broadcast stage, Sec. 3.3): aggregated entries whose
    mask bit is clear never arrived and count as zero.  mask: padded_len(n)/32 uint32 words."""
    a = _arr(agg, np.float32)
    m = _arr(mask, np.uint32)
    assert a.size == padded_len(n, block_log2) and m.size == a.size // 32
    if out_dtype is not None and np.dtype(out_dtype) == np.uint16:
        out = np.empty(n, np.uint16)
        fn = "orc_rht_decode_masked_bf16"
    else:
        out = np.empty(n, np.float32)
        fn = "orc_rht_decode_masked_f32"
    getattr(_load(), fn)(_ptr(a), _ptr(m), n, block_log2, seed, base_index, _ptr(out))
    return out


def received_total(count) -> int:
    """Sec. 3.4 loss monitoring: total number of (worker, entry) arrivals in the counts of one shard."""
    c = _arr(count, np.uint8)
    return int(_load().orc_received_total(_ptr(c), c.size))


def loss_decision(received_total: int, N: int, shard_len: int, transform_on_loss: float, skip_loss: float,
                  halt_loss: float, prev_transform_on: bool):
    """Sec. 3.4 (skip the update or halt above a loss threshold) and Sec. 3.2.1 (the transform goes on
    above 2 % loss and stays on).  loss = 1 - received / (N * shard_len), compared as exact rationals.
    Returns (action, transform_on, loss) with action 0 = apply, 1 = skip, 2 = halt."""
    from fractions import Fraction
    sent = N * shard_len
    assert 0 <= received_total <= sent and sent > 0
    loss = 1 - Fraction(received_total, sent)
    action = 2 if loss > Fraction(halt_loss) else (1 if loss > Fraction(skip_loss) else 0)
    return action, bool(prev_transform_on or loss > Fraction(transform_on_loss)), float(loss)


def masked_reduce_pairs(sums, counts, masks):
    """Second level of hierarchical 2D TAR (Sec. 3.1.2, App. A): combine the groups' (sum, count)
    partial aggregates that arrived.  sums [G, L] fp32, counts [G, L] uint8, masks [G, L/32]."""
    s = _arr(sums, np.float32)
    c = _arr(counts, np.uint8)
    m = _arr(masks, np.uint32)
    G, Ln = s.shape
    assert c.shape == (G, Ln) and m.shape == (G, Ln // 32) and Ln % 32 == 0
    total = np.empty(Ln, np.float32)
    count = np.empty(Ln, np.uint8)
    _load().orc_masked_reduce_pairs(_ptr(s), _ptr(c), _ptr(m), G, Ln, _ptr(total), _ptr(count))
    return total, count


def fused_path(grads, masks, block_log2: int, seed: int, base_index: int = 0):
    """Encode each worker's raw slice, masked sum and count, mean, decode: the composition of the
    steps above with every boundary rounding kept.  grads [N, L] float32 or uint16 (bf16 bits).
    Returns (decoded [L], count uint8 [L])."""
    g = np.ascontiguousarray(grads)
    m = _arr(masks, np.uint32)
    N, Ln = g.shape
    assert Ln % (1 << block_log2) == 0 and m.shape == (N, Ln // 32)
    out = np.empty(Ln, g.dtype)
    count = np.empty(Ln, np.uint8)
    fn = "orc_fused_path_f32" if g.dtype == np.float32 else "orc_fused_path_bf16"
    assert g.dtype in (np.float32, np.uint16)
    getattr(_load(), fn)(_ptr(g), _ptr(m), N, Ln, block_log2, seed, base_index, _ptr(out), _ptr(count))
    return out, count
