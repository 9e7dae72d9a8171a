// Host-side table of kernel launchers, one table per block-size class.  Each class is compiled in
// its own translation unit (inst.hip with -DOR_K=<class>) so the classes build in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include "rht_kernels.hpp"

namespace orhost {

typedef hipError_t (*launch_fn)(const ordev::PathArgs&, unsigned long long units, hipStream_t);

struct KernelTable {
  int tile_log2;              // entries per workgroup tile
  launch_fn encode_f32, encode_bf16;
  launch_fn decode_f32, decode_bf16;                    // input: fp32 mean
  launch_fn finalize_decode_f32, finalize_decode_bf16;  // input: fp32 sum + u8 count
  launch_fn reduce_decode_f32, reduce_decode_bf16;      // null when a block spans several tiles
  launch_fn fused_f32, fused_bf16;                      // decode fused in when a block is one tile, else stops at the mean
};

// class 0 serves every block_log2 <= 10; classes 11..16 serve exactly that block_log2
const KernelTable* table_for_class(int cls);

}  // namespace orhost
