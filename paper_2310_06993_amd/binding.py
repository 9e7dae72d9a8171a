"""Thin ctypes binding of liboptireduce_hip.so: argument marshalling only.

Every function has the name and argument order of its C entry point in include/optireduce.h and
takes torch tensors that already live on the GPU (torch is used for device memory and streams,
nothing else).  A non-zero status raises OptiReduceError.  There is no CPU fallback: if the
library is not built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "liboptireduce_hip.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(
        "liboptireduce_hip.so is not built (%s); run `python -m paper_2310_06993_amd.build`" % _LIB_PATH)
lib = C.CDLL(_LIB_PATH)

_u64, _int, _p, _sz = C.c_uint64, C.c_int, C.c_void_p, C.c_size_t

OR_OK = 0
OR_MIN_LOG2, OR_MAX_LOG2, OR_MAX_WORKERS = 5, 16, 255

_SIGS = {
    "or_padded_len": (_u64, [_u64, _int]),
    "or_workspace_bytes": (_sz, [_u64, _int]),
    "or_status_string": (C.c_char_p, [_int]),
    "or_version": (_int, []),
    "or_last_hip_error": (_int, []),
    "or_time_next_call": (_int, [_p, _p]),
    "or_rht_encode": (_int, [_p, _u64, _int, _u64, _p, _p]),
    "or_rht_encode_at": (_int, [_p, _u64, _int, _u64, _u64, _p, _p]),
    "or_rht_encode_bf16": (_int, [_p, _u64, _int, _u64, _u64, _p, _p]),
    "or_masked_reduce": (_int, [_p, _p, _int, _u64, _p, _p, _p]),
    "or_masked_reduce_bf16": (_int, [_p, _p, _int, _u64, _p, _p, _p]),
    "or_rht_decode": (_int, [_p, _u64, _int, _u64, _p, _p]),
    "or_rht_decode_at": (_int, [_p, _u64, _int, _u64, _u64, _p, _p]),
    "or_rht_decode_bf16": (_int, [_p, _u64, _int, _u64, _u64, _p, _p]),
    "or_finalize_decode": (_int, [_p, _p, _u64, _int, _u64, _u64, _p, _p]),
    "or_finalize_decode_bf16": (_int, [_p, _p, _u64, _int, _u64, _u64, _p, _p]),
    "or_reduce_decode": (_int, [_p, _p, _int, _u64, _int, _u64, _u64, _p, _p, _p, _sz, _p]),
    "or_reduce_decode_bf16": (_int, [_p, _p, _int, _u64, _int, _u64, _u64, _p, _p, _p, _sz, _p]),
    "or_fused_path": (_int, [_p, _p, _int, _u64, _int, _u64, _u64, _p, _p, _p, _sz, _p]),
    "or_fused_path_bf16": (_int, [_p, _p, _int, _u64, _int, _u64, _u64, _p, _p, _p, _sz, _p]),
    "or_fused_path_bf16_static": (_int, [_p, _p, _int, _u64, _int, _u64, _u64, _p, _p, _p]),
    "or_fused_path_batched": (_int, [_p, _int, _int, _int, _int, _p, _sz, _p]),
    "or_fused_path_batched_monitored": (_int, [_p, _int, _int, _int, _int, _p, _p, _sz, _p]),
    "or_reduce_decode_batched": (_int, [_p, _int, _int, _int, _int, _p, _p, _sz, _p]),
    "or_masked_reduce_batched": (_int, [_p, _int, _int, _int, _p]),
    "or_finalize_decode_batched": (_int, [_p, _int, _int, _int, _p]),
    "or_finalize": (_int, [_p, _p, _u64, _p, _p]),
    "or_finalize_bf16": (_int, [_p, _p, _u64, _p, _p]),
    "or_received_total": (_int, [_p, _u64, _p, _p]),
    "or_loss_decision": (_int, [_u64, _int, _u64, _p, _int, _p, _p, _p]),
    "or_rht_decode_masked": (_int, [_p, _p, _u64, _int, _u64, _u64, _p, _p]),
    "or_rht_decode_masked_bf16": (_int, [_p, _p, _u64, _int, _u64, _u64, _p, _p]),
    "or_masked_reduce_pairs": (_int, [_p, _p, _p, _int, _u64, _p, _p, _p]),
}


OR_ACT_APPLY, OR_ACT_SKIP, OR_ACT_HALT = 0, 1, 2
OR_DEFAULT_TRANSFORM_ON_LOSS = 0.02


class or_loss_policy(C.Structure):
    _fields_ = [("transform_on_loss", C.c_double), ("skip_loss", C.c_double), ("halt_loss", C.c_double)]


class or_bucket(C.Structure):
    _fields_ = [("grads", _p), ("masks", _p), ("out", _p), ("count_out", _p),
                ("shard_len", _u64), ("seed", _u64), ("base_index", _u64)]


class or_stage_bucket(C.Structure):
    _fields_ = [("shards", _p), ("masks", _p), ("sum", _p), ("count", _p), ("out", _p),
                ("shard_len", _u64), ("seed", _u64), ("base_index", _u64)]


for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args


class OptiReduceError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, lib.or_status_string(status).decode()))


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("liboptireduce_hip takes device tensors")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(status, where):
    if status != OR_OK:
        raise OptiReduceError(status, where)


def or_padded_len(n: int, block_log2: int) -> int:
    return int(lib.or_padded_len(n, block_log2))


def or_workspace_bytes(shard_len: int, block_log2: int) -> int:
    return int(lib.or_workspace_bytes(shard_len, block_log2))


def or_version() -> int:
    return int(lib.or_version())


def or_time_next_call(start_event, stop_event):
    """start_event / stop_event: raw hipEvent_t handles (ints) or None."""
    _check(lib.or_time_next_call(start_event, stop_event), "or_time_next_call")


def or_rht_encode(grad, n, block_log2, seed, out, stream=None):
    _check(lib.or_rht_encode(_ptr(grad), n, block_log2, seed, _ptr(out), _stream(stream)), "or_rht_encode")


def or_rht_encode_at(grad, n, block_log2, seed, base_index, out, stream=None):
    _check(lib.or_rht_encode_at(_ptr(grad), n, block_log2, seed, base_index, _ptr(out), _stream(stream)),
           "or_rht_encode_at")


def or_rht_encode_bf16(grad, n, block_log2, seed, base_index, out, stream=None):
    _check(lib.or_rht_encode_bf16(_ptr(grad), n, block_log2, seed, base_index, _ptr(out), _stream(stream)),
           "or_rht_encode_bf16")


def or_masked_reduce(shards, masks, N, shard_len, sum_out, count_out, stream=None):
    _check(lib.or_masked_reduce(_ptr(shards), _ptr(masks), N, shard_len, _ptr(sum_out), _ptr(count_out),
                                _stream(stream)), "or_masked_reduce")


def or_masked_reduce_bf16(shards, masks, N, shard_len, sum_out, count_out, stream=None):
    _check(lib.or_masked_reduce_bf16(_ptr(shards), _ptr(masks), N, shard_len, _ptr(sum_out), _ptr(count_out),
                                     _stream(stream)), "or_masked_reduce_bf16")


def or_rht_decode(agg, n, block_log2, seed, out, stream=None):
    _check(lib.or_rht_decode(_ptr(agg), n, block_log2, seed, _ptr(out), _stream(stream)), "or_rht_decode")


def or_rht_decode_at(agg, n, block_log2, seed, base_index, out, stream=None):
    _check(lib.or_rht_decode_at(_ptr(agg), n, block_log2, seed, base_index, _ptr(out), _stream(stream)),
           "or_rht_decode_at")


def or_rht_decode_bf16(agg, n, block_log2, seed, base_index, out, stream=None):
    _check(lib.or_rht_decode_bf16(_ptr(agg), n, block_log2, seed, base_index, _ptr(out), _stream(stream)),
           "or_rht_decode_bf16")


def or_finalize_decode(total, count, n, block_log2, seed, base_index, out, stream=None):
    _check(lib.or_finalize_decode(_ptr(total), _ptr(count), n, block_log2, seed, base_index, _ptr(out),
                                  _stream(stream)), "or_finalize_decode")


def or_finalize_decode_bf16(total, count, n, block_log2, seed, base_index, out, stream=None):
    _check(lib.or_finalize_decode_bf16(_ptr(total), _ptr(count), n, block_log2, seed, base_index, _ptr(out),
                                       _stream(stream)), "or_finalize_decode_bf16")


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _ptr(workspace), workspace.numel() * workspace.element_size()


def or_reduce_decode(shards, masks, N, shard_len, block_log2, seed, base_index, out, count_out=None,
                     workspace=None, stream=None):
    w, wb = _ws(workspace)
    _check(lib.or_reduce_decode(_ptr(shards), _ptr(masks), N, shard_len, block_log2, seed, base_index, _ptr(out),
                                _ptr(count_out), w, wb, _stream(stream)), "or_reduce_decode")


def or_reduce_decode_bf16(shards, masks, N, shard_len, block_log2, seed, base_index, out, count_out=None,
                          workspace=None, stream=None):
    w, wb = _ws(workspace)
    _check(lib.or_reduce_decode_bf16(_ptr(shards), _ptr(masks), N, shard_len, block_log2, seed, base_index,
                                     _ptr(out), _ptr(count_out), w, wb, _stream(stream)), "or_reduce_decode_bf16")


def or_fused_path(grads, masks, N, shard_len, block_log2, seed, base_index, out, count_out=None, workspace=None,
                  stream=None):
    w, wb = _ws(workspace)
    _check(lib.or_fused_path(_ptr(grads), _ptr(masks), N, shard_len, block_log2, seed, base_index, _ptr(out),
                             _ptr(count_out), w, wb, _stream(stream)), "or_fused_path")


def or_fused_path_bf16(grads, masks, N, shard_len, block_log2, seed, base_index, out, count_out=None,
                       workspace=None, stream=None):
    w, wb = _ws(workspace)
    _check(lib.or_fused_path_bf16(_ptr(grads), _ptr(masks), N, shard_len, block_log2, seed, base_index, _ptr(out),
                                  _ptr(count_out), w, wb, _stream(stream)), "or_fused_path_bf16")


OR_STATIC_MAX_SHARD_LEN = 4194304


def or_fused_path_bf16_static(grads, masks, N, shard_len, block_log2, seed, base_index, out, count_out=None,
                              stream=None):
    _check(lib.or_fused_path_bf16_static(_ptr(grads), _ptr(masks), N, shard_len, block_log2, seed, base_index,
                                         _ptr(out), _ptr(count_out), _stream(stream)), "or_fused_path_bf16_static")


def make_buckets(items):
    """items: iterable of (grads, masks, out, count_out_or_None, shard_len, seed, base_index) with device
    tensors -> a host array of or_bucket that or_fused_path_batched can take (reusable across calls)."""
    items = list(items)
    arr = (or_bucket * len(items))()
    for j, (g, m, o, c, L, seed, base) in enumerate(items):
        arr[j] = or_bucket(_ptr(g), _ptr(m), _ptr(o), _ptr(c), L, seed, base)
    return arr


def or_fused_path_batched(buckets, n_buckets, N, block_log2, bf16, workspace=None, stream=None):
    w, wb = _ws(workspace)
    _check(lib.or_fused_path_batched(C.cast(buckets, _p), n_buckets, N, block_log2, int(bool(bf16)), w, wb,
                                     _stream(stream)), "or_fused_path_batched")


def or_fused_path_batched_monitored(buckets, n_buckets, N, block_log2, bf16, totals, workspace=None, stream=None):
    """totals: an int64 device tensor of n_buckets entries, or None."""
    w, wb = _ws(workspace)
    _check(lib.or_fused_path_batched_monitored(C.cast(buckets, _p), n_buckets, N, block_log2, int(bool(bf16)),
                                               _ptr(totals), w, wb, _stream(stream)),
           "or_fused_path_batched_monitored")


def or_reduce_decode_batched(buckets, n_buckets, N, block_log2, bf16, totals=None, workspace=None, stream=None):
    w, wb = _ws(workspace)
    _check(lib.or_reduce_decode_batched(C.cast(buckets, _p), n_buckets, N, block_log2, int(bool(bf16)),
                                        _ptr(totals), w, wb, _stream(stream)), "or_reduce_decode_batched")


def make_stage_buckets(items):
    """items: iterable of (shards, masks, sum, count, out, shard_len, seed, base_index) with device tensors
    (or None where the call ignores the field) -> a host array of or_stage_bucket."""
    items = list(items)
    arr = (or_stage_bucket * len(items))()
    for j, (sh, m, t, c, o, L, seed, base) in enumerate(items):
        arr[j] = or_stage_bucket(_ptr(sh), _ptr(m), _ptr(t), _ptr(c), _ptr(o), L, seed, base)
    return arr


def or_masked_reduce_batched(buckets, n_buckets, N, bf16, stream=None):
    _check(lib.or_masked_reduce_batched(C.cast(buckets, _p), n_buckets, N, int(bool(bf16)), _stream(stream)),
           "or_masked_reduce_batched")


def or_finalize_decode_batched(buckets, n_buckets, block_log2, bf16, stream=None):
    _check(lib.or_finalize_decode_batched(C.cast(buckets, _p), n_buckets, block_log2, int(bool(bf16)),
                                          _stream(stream)), "or_finalize_decode_batched")


def or_finalize(total, count, shard_len, mean_out, stream=None):
    _check(lib.or_finalize(_ptr(total), _ptr(count), shard_len, _ptr(mean_out), _stream(stream)), "or_finalize")


def or_finalize_bf16(total, count, shard_len, mean_out, stream=None):
    _check(lib.or_finalize_bf16(_ptr(total), _ptr(count), shard_len, _ptr(mean_out), _stream(stream)),
           "or_finalize_bf16")


def or_received_total(count, shard_len, total_out, stream=None):
    """total_out: a one-element int64 device tensor."""
    _check(lib.or_received_total(_ptr(count), shard_len, _ptr(total_out), _stream(stream)), "or_received_total")


def or_loss_decision(received_total, N, shard_len, policy, prev_transform_on):
    """Host arithmetic only.  policy: an or_loss_policy.  Returns (action, transform_on, loss)."""
    act, ton, loss = C.c_int(), C.c_int(), C.c_double()
    _check(lib.or_loss_decision(int(received_total), N, shard_len, C.byref(policy), int(bool(prev_transform_on)),
                                C.byref(act), C.byref(ton), C.byref(loss)), "or_loss_decision")
    return act.value, ton.value, loss.value


def or_rht_decode_masked(agg, mask, n, block_log2, seed, base_index, out, stream=None):
    _check(lib.or_rht_decode_masked(_ptr(agg), _ptr(mask), n, block_log2, seed, base_index, _ptr(out),
                                    _stream(stream)), "or_rht_decode_masked")


def or_rht_decode_masked_bf16(agg, mask, n, block_log2, seed, base_index, out, stream=None):
    _check(lib.or_rht_decode_masked_bf16(_ptr(agg), _ptr(mask), n, block_log2, seed, base_index, _ptr(out),
                                         _stream(stream)), "or_rht_decode_masked_bf16")


def or_masked_reduce_pairs(sums, counts, masks, G, shard_len, sum_out, count_out, stream=None):
    _check(lib.or_masked_reduce_pairs(_ptr(sums), _ptr(counts), _ptr(masks), G, shard_len, _ptr(sum_out),
                                      _ptr(count_out), _stream(stream)), "or_masked_reduce_pairs")
