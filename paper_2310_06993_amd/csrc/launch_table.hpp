// Host-side table of kernel launchers, one table per block-size class.  Each class is compiled in
// its own translation unit (inst.hip with -DOR_K=<class>) so the classes build in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include "rht_kernels.hpp"

namespace orhost {

// `pos`: LAUNCH_FIRST / LAUNCH_LAST mark the first / last kernel an entry point enqueues (both for a
// single-kernel call); they select which of the caller's timing events, if armed, ride on the launch.
enum { LAUNCH_FIRST = 1, LAUNCH_LAST = 2, LAUNCH_ONLY = 3 };
typedef hipError_t (*launch_fn)(const ordev::PathArgs&, unsigned long long units, hipStream_t, int pos);

// Timing events armed by or_time_next_call for the calling thread (null when not armed).
struct TimingEvents { hipEvent_t start, stop; };
TimingEvents& timing_events();

// Launch with the armed events attached to the dispatch itself (they then carry the kernel's own begin
// and end timestamps, as a profiler would see them), or plainly when none are armed.
template <class Kernel, class... Args>
inline hipError_t launch_kernel(Kernel kernel, dim3 grid, dim3 block, hipStream_t s, int pos, Args... args) {
  TimingEvents& t = timing_events();
  hipEvent_t e0 = (pos & LAUNCH_FIRST) ? t.start : nullptr;
  hipEvent_t e1 = (pos & LAUNCH_LAST) ? t.stop : nullptr;
  if (e0 || e1) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, e0, e1, 0, args...);
  else hipLaunchKernelGGL(kernel, grid, block, 0, s, args...);
  return hipGetLastError();
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
};

// class 0 serves every block_log2 <= 10; classes 11..16 serve exactly that block_log2
const KernelTable* table_for_class(int cls);

}  // namespace orhost
