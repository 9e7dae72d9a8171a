// Host-side table of kernel launchers, one table per block-size class.  Each class is compiled in
// its own translation unit (inst.hip with -DOR_K=<class>) so the classes build in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <tuple>
#include <utility>
#include "rht_kernels.hpp"

namespace orhost {

// `pos`: LAUNCH_FIRST / LAUNCH_LAST mark the first / last kernel an entry point enqueues (both for a
// single-kernel call); they select which of the caller's timing events, if armed, ride on the launch.
enum { LAUNCH_FIRST = 1, LAUNCH_LAST = 2, LAUNCH_ONLY = 3 };
typedef hipError_t (*launch_fn)(const ordev::PathArgs&, unsigned long long units, hipStream_t, int pos);

// Timing events armed by or_time_next_call for the calling thread (null when not armed).
struct TimingEvents { hipEvent_t start, stop; };
TimingEvents& timing_events();

template <class Tuple, size_t... I>
inline void fill_argv(Tuple& held, void** argv, std::index_sequence<I...>) {
  ((argv[I] = (void*)&std::get<I>(held)), ...);
}

// Launch with the armed events attached to the dispatch itself (they then carry the kernel's own begin
// and end timestamps, as a profiler would see them), or plainly when none are armed.  The status is the
// one the launch call returns: an error that some earlier call left behind on this thread is neither
// reported as this launch's nor cleared.
template <class... Params, class... Args>
inline hipError_t launch_kernel(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t s, int pos, Args... args) {
  static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
  TimingEvents& t = timing_events();
  hipEvent_t e0 = (pos & LAUNCH_FIRST) ? t.start : nullptr;
  hipEvent_t e1 = (pos & LAUNCH_LAST) ? t.stop : nullptr;
  std::tuple<Params...> held(args...);   // converted to the kernel's own parameter types
  void* argv[sizeof...(Params)];
  fill_argv(held, argv, std::index_sequence_for<Params...>{});
  if (e0 || e1) return hipExtLaunchKernel((const void*)kernel, grid, block, argv, 0, s, e0, e1, 0);
  return hipLaunchKernel((const void*)kernel, grid, block, argv, 0, s);
}

typedef hipError_t (*batch_fn)(const ordev::BatchArgs&, unsigned long long units, hipStream_t, int pos);

struct KernelTable {
  int tile_log2;              // entries per workgroup tile
  launch_fn encode_f32, encode_bf16;
  launch_fn decode_f32, decode_bf16;                    // input: fp32 mean
  launch_fn finalize_decode_f32, finalize_decode_bf16;  // input: fp32 sum + u8 count
  launch_fn decode_masked_f32, decode_masked_bf16;      // input: fp32 mean + received bits of the second stage
  launch_fn reduce_decode_f32, reduce_decode_bf16;      // null when a block spans several tiles
  launch_fn fused_f32, fused_bf16;                      // decode fused in when a block is one tile, else stops at the mean
  batch_fn fused_batched_f32, fused_batched_bf16;       // null when a block spans several tiles
  batch_fn reduce_decode_batched_f32, reduce_decode_batched_bf16;       // likewise
  batch_fn finalize_decode_batched_f32, finalize_decode_batched_bf16;   // likewise
};

// class 0 serves every block_log2 <= 10; classes 11..16 serve exactly that block_log2
const KernelTable* table_for_class(int cls);

}  // namespace orhost
