// C ABI of liboptireduce_hip: argument checks and kernel dispatch.  Semantics are stated in
// include/optireduce.h; nothing here allocates or synchronises.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <mutex>

#include "../../include/optireduce.h"
#include "launch_table.hpp"

namespace orhost {
extern const KernelTable or_kernel_table_0, or_kernel_table_11, or_kernel_table_12, or_kernel_table_13,
    or_kernel_table_14, or_kernel_table_15, or_kernel_table_16;

TimingEvents& timing_events() {
  static thread_local TimingEvents t = {nullptr, nullptr};
  return t;
}

const KernelTable* table_for_class(int cls) {
  switch (cls) {
    case 0: return &or_kernel_table_0;
    case 11: return &or_kernel_table_11;
    case 12: return &or_kernel_table_12;
    case 13: return &or_kernel_table_13;
    case 14: return &or_kernel_table_14;
    case 15: return &or_kernel_table_15;
    case 16: return &or_kernel_table_16;
    default: return nullptr;
  }
}
}  // namespace orhost

namespace {
using ordev::PathArgs;
using ordev::u64;

thread_local int g_last_hip_error = 0;

// ------------------------------------------------------------------ streaming masked sum + count
// Sec. 3.1.1 aggregation with no transform around it: each lane owns VEC consecutive entries (16
// bytes of one worker's shard), reads the VEC mask bits of every worker and adds under select.
#ifndef OR_NT_REDUCE
#define OR_NT_REDUCE true
#endif
template <class Wire, int VEC>
__device__ __forceinline__ void masked_reduce_at(const Wire* __restrict__ shards, const uint32_t* __restrict__ masks,
                                                 int N, u64 L, float* __restrict__ sum_out,
                                                 uint8_t* __restrict__ count_out, u64 e) {
  if (e >= L) return;
  typedef Wire vec_t __attribute__((ext_vector_type(VEC)));
  const u64 words = L >> 5;
  float acc[VEC];
  uint32_t cnt[VEC];
#pragma unroll
  for (int j = 0; j < VEC; ++j) { acc[j] = 0.0f; cnt[j] = 0; }
  const int sh = (int)(e & 31);
  int i = 0;
  for (; i + 4 <= N; i += 4) {
    vec_t x[4];
    uint32_t m[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      x[u] = OR_NT_REDUCE ? __builtin_nontemporal_load((const vec_t*)(shards + (u64)(i + u) * L + e))
                          : *(const vec_t*)(shards + (u64)(i + u) * L + e);
      m[u] = masks[(u64)(i + u) * words + (e >> 5)] >> sh;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        const bool got = (m[u] >> j) & 1u;
        float f;
        if constexpr (sizeof(Wire) == 4) f = x[u][j]; else f = __builtin_bit_cast(float, (uint32_t)x[u][j] << 16);
        acc[j] += got ? f : 0.0f;
        cnt[j] += got ? 1u : 0u;
      }
  }
  for (; i < N; ++i) {
    vec_t x = OR_NT_REDUCE ? __builtin_nontemporal_load((const vec_t*)(shards + (u64)i * L + e))
                           : *(const vec_t*)(shards + (u64)i * L + e);
    uint32_t m = masks[(u64)i * words + (e >> 5)] >> sh;
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      const bool got = (m >> j) & 1u;
      float f;
      if constexpr (sizeof(Wire) == 4) f = x[j]; else f = __builtin_bit_cast(float, (uint32_t)x[j] << 16);
      acc[j] += got ? f : 0.0f;
      cnt[j] += got ? 1u : 0u;
    }
  }
  // nontemporal: the results are not read again here and reads dominate the traffic
  typedef float f4 __attribute__((ext_vector_type(4)));
#pragma unroll
  for (int j = 0; j < VEC; j += 4)
    __builtin_nontemporal_store(f4{acc[j], acc[j + 1], acc[j + 2], acc[j + 3]}, (f4*)(sum_out + e + j));
#pragma unroll
  for (int j = 0; j < VEC; j += 4)
    __builtin_nontemporal_store(cnt[j] | (cnt[j + 1] << 8) | (cnt[j + 2] << 16) | (cnt[j + 3] << 24),
                                (uint32_t*)(count_out + e + j));
}

template <class Wire, int VEC>
__global__ __launch_bounds__(256) void k_masked_reduce(const Wire* __restrict__ shards,
                                                       const uint32_t* __restrict__ masks, int N, u64 L,
                                                       float* __restrict__ sum_out, uint8_t* __restrict__ count_out) {
  masked_reduce_at<Wire, VEC>(shards, masks, N, L, sum_out, count_out, ((u64)blockIdx.x * 256 + threadIdx.x) * VEC);
}

// several buckets in one launch (a 25 MiB bucket is a few hundred workgroups here): descriptors in the kernel
// arguments; workgroup x serves entries of bucket j from (x - start[j]) * 256 * VEC on
struct ReduceBucket {
  const void* shards;
  const uint32_t* masks;
  float* sum;
  uint8_t* count;
  u64 L;
};
struct ReduceBatch {
  int n, N;
  uint32_t start[ordev::kMaxBatch + 1];
  ReduceBucket b[ordev::kMaxBatch];
};
static_assert(sizeof(ReduceBatch) <= 4096, "kernel arguments are limited to 4 KB");
template <class Wire, int VEC>
__global__ __launch_bounds__(256) void k_masked_reduce_batched(ReduceBatch rb) {
  const uint32_t x = blockIdx.x;
  int j = 0;
  while (j + 1 < rb.n && rb.start[j + 1] <= x) ++j;
  masked_reduce_at<Wire, VEC>((const Wire*)rb.b[j].shards, rb.b[j].masks, rb.N, rb.b[j].L, rb.b[j].sum, rb.b[j].count,
                              ((u64)(x - rb.start[j]) * 256 + threadIdx.x) * VEC);
}

template <class Wire, int VEC>
hipError_t launch_masked_reduce(const void* shards, const uint32_t* masks, int N, u64 L, float* sum_out,
                                uint8_t* count_out, hipStream_t s, int pos) {
  if (L == 0) return hipSuccess;
  const u64 threads = (L + VEC - 1) / VEC;
  const u64 blocks = (threads + 255) / 256;
  if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
  return orhost::launch_kernel(k_masked_reduce<Wire, VEC>, dim3((unsigned)blocks), dim3(256), s, pos,
                               (const Wire*)shards, masks, N, L, sum_out, count_out);
}

// ------------------------------------------------------------------ small streaming kernels
// mean = sum / count, 0 where count is 0 (Sec. 3.1.1 "averages" over what arrived); 4 entries per lane
template <class Out>
__global__ __launch_bounds__(256) void k_finalize(const float* __restrict__ sum, const uint8_t* __restrict__ count, u64 L,
                                                  Out* __restrict__ mean) {
  const u64 e = ((u64)blockIdx.x * 256 + threadIdx.x) * 4;
  if (e >= L) return;
  typedef float f4 __attribute__((ext_vector_type(4)));
  const f4 s4 = *(const f4*)(sum + e);
  const uint32_t c4 = *(const uint32_t*)(count + e);
  float m[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float c = (float)((c4 >> (8 * j)) & 0xFFu);
    m[j] = c > 0.0f ? s4[j] / c : 0.0f;
  }
  if constexpr (sizeof(Out) == 4) {
    *(f4*)(mean + e) = f4{m[0], m[1], m[2], m[3]};
  } else {
    typedef uint16_t h4 __attribute__((ext_vector_type(4)));
    h4 h;
#pragma unroll
    for (int j = 0; j < 4; ++j) h[j] = __builtin_bit_cast(uint16_t, (__bf16)m[j]);
    *(h4*)(mean + e) = h;
  }
}

__global__ void k_zero_u64(unsigned long long* p) { *p = 0; }
__global__ __launch_bounds__(256) void k_zero_u64n(unsigned long long* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Sign bits of n_counters * 128 consecutive entries as a table: the Philox output for counter
// first_counter + c, 16 bytes, at tab + 16 c -- so bit j of 64-bit word w is the sign of entry 64 w + j
// counted from the first entry.  The fused kernels for blocks above 2^14 read it with scalar loads.
__global__ __launch_bounds__(256) void k_sign_table(uint4* __restrict__ tab, u64 seed, u64 first_counter,
                                                    u64 n_counters, unsigned* __restrict__ flags, u64 n_flag_words) {
  const u64 c = (u64)blockIdx.x * 256 + threadIdx.x;
  if (c < n_flag_words) flags[c] = 0;   // the words of the pair hand-over of the bf16 kernel for 2^16 blocks
  if (c >= n_counters) return;
  const u64 ctr = first_counter + c;
  const ordev::u32x4 w =
      ordev::philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
  tab[c] = make_uint4(w.a, w.b, w.c, w.d);
}

// Sec. 3.4 loss monitoring: total of the received counts of a shard (16 counts per lane, byte sums
// with v_sad_u8, one 64-bit atomic per wavefront)
__global__ __launch_bounds__(256) void k_received_total(const uint8_t* __restrict__ count, u64 L,
                                                        unsigned long long* __restrict__ total) {
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  uint32_t acc = 0;
  for (u64 e = ((u64)blockIdx.x * 256 + threadIdx.x) * 16; e < L; e += (u64)gridDim.x * 256 * 16) {
    if (e + 16 <= L) {
      const u4 c = *(const u4*)(count + e);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_sad_u8(c[j], 0u, acc);
    } else {
      for (u64 i = e; i < L; ++i) acc += count[i];
    }
  }
  unsigned long long w = acc;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) w += __shfl_xor(w, o, 64);
  if ((threadIdx.x & 63) == 0 && w) atomicAdd(total, w);
}

// Second level of hierarchical 2D TAR (Sec. 3.1.2, App. A): sums with sums, counts with counts, over
// the groups whose partial aggregate arrived; 4 entries per lane
__global__ __launch_bounds__(256) void k_masked_reduce_pairs(const float* __restrict__ sums,
                                                             const uint8_t* __restrict__ counts,
                                                             const uint32_t* __restrict__ masks, int G, u64 L,
                                                             float* __restrict__ sum_out,
                                                             uint8_t* __restrict__ count_out) {
  const u64 e = ((u64)blockIdx.x * 256 + threadIdx.x) * 4;
  if (e >= L) return;
  typedef float f4 __attribute__((ext_vector_type(4)));
  const u64 words = L >> 5;
  const int sh = (int)(e & 31);
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  uint32_t cnt[4] = {0, 0, 0, 0};
  for (int g = 0; g < G; ++g) {
    // read once: nontemporal, as in k_masked_reduce
    const f4 x = __builtin_nontemporal_load((const f4*)(sums + (u64)g * L + e));
    const uint32_t c4 = __builtin_nontemporal_load((const uint32_t*)(counts + (u64)g * L + e));
    const uint32_t m = masks[(u64)g * words + (e >> 5)] >> sh;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool got = (m >> j) & 1u;
      acc[j] += got ? x[j] : 0.0f;
      cnt[j] += got ? ((c4 >> (8 * j)) & 0xFFu) : 0u;
    }
  }
  __builtin_nontemporal_store(f4{acc[0], acc[1], acc[2], acc[3]}, (f4*)(sum_out + e));
  __builtin_nontemporal_store((cnt[0] & 0xFFu) | ((cnt[1] & 0xFFu) << 8) | ((cnt[2] & 0xFFu) << 16) | (cnt[3] << 24),
                              (uint32_t*)(count_out + e));
}

// ------------------------------------------------------------------ checks
bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }
bool valid_k(int k) { return k >= OR_MIN_LOG2 && k <= OR_MAX_LOG2; }
int class_of(int k) { return k <= 10 ? 0 : k; }

bool ranges_overlap(const void* a, u64 abytes, const void* b, u64 bbytes) {
  uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a0 < b0 + bbytes && b0 < a0 + abytes;
}

// armed timing events serve exactly one entry-point call, whatever its outcome
struct DisarmOnExit {
  ~DisarmOnExit() { orhost::timing_events() = {nullptr, nullptr}; }
};

or_status finish(hipError_t e) {
  if (e == hipSuccess) return OR_OK;
  g_last_hip_error = (int)e;
  return OR_ERR_HIP;
}

u64 padded(u64 n, int k) {
  const u64 B = (u64)1 << k;
  return (n + B - 1) / B * B;
}

// number of leading tiles that lie, together with every other tile of their transform block, wholly inside
// the first n entries (those need no bounds checks)
u64 full_units(u64 n, int k, int tile_log2) {
  const int group_log2 = k > tile_log2 ? k : tile_log2;   // a block above 2^14 spans 2^(k-14) tiles
  return (n >> group_log2) << (group_log2 - tile_log2);
}

float scale_of(int k) { return (float)(1.0 / sqrt((double)((u64)1 << k))); }

or_status check_base(int k, u64 base) {
  const u64 B = (u64)1 << k;
  const u64 q = B > 128 ? B : 128;
  return (base % q) ? OR_ERR_SHAPE : OR_OK;
}

// vector transforms: `in_es`/`out_es` are element sizes; the side of length n_pad is the encoded one
or_status check_transform(const void* in, u64 in_len, int in_es, void* out, u64 out_len, int out_es, int k, u64 base) {
  if (!valid_k(k)) return OR_ERR_BLOCK;
  if (check_base(k, base)) return OR_ERR_SHAPE;
  if (in_len == 0 && out_len == 0) return OR_OK;
  if (!in || !out) return OR_ERR_NULL;
  if (!aligned(in, 16) || !aligned(out, 16)) return OR_ERR_ALIGN;
  if (in_len > ((u64)1 << 46) || out_len > ((u64)1 << 46)) return OR_ERR_SHAPE;
  if (ranges_overlap(in, in_len * in_es, out, out_len * out_es)) {
    // every workgroup reads the whole of its tile (or block of tiles) before it writes any of it
    const bool exact_in_place = (in == out) && in_len == out_len && in_es == out_es;
    if (!exact_in_place) return OR_ERR_SHAPE;
  }
  return OR_OK;
}

template <class T>
or_status encode_impl(const T* grad, u64 n, int k, u64 seed, u64 base, T* out, void* stream, bool bf16) {
  DisarmOnExit disarm;
  const u64 n_pad = valid_k(k) ? padded(n, k) : 0;
  if (or_status s = check_transform(grad, n, sizeof(T), out, n_pad, sizeof(T), k, base)) return s;
  if (n == 0) return OR_OK;
  const orhost::KernelTable* t = orhost::table_for_class(class_of(k));
  PathArgs a = {};
  a.in = grad; a.out = out; a.n = n; a.n_pad = n_pad; a.seed = seed; a.base = base; a.k = k; a.scale = scale_of(k);
  const u64 units = (n_pad + ((u64)1 << t->tile_log2) - 1) >> t->tile_log2;
  a.unit0 = full_units(n, k, t->tile_log2);   // tiles whose whole block lies inside the n valid entries
  return finish((bf16 ? t->encode_bf16 : t->encode_f32)(a, units, (hipStream_t)stream, orhost::LAUNCH_ONLY));
}

template <class T>
or_status decode_impl(const float* agg, const uint8_t* count, bool finalize, u64 n, int k, u64 seed, u64 base, T* out,
                      void* stream, bool bf16, const uint32_t* stage2_mask = nullptr, bool masked = false) {
  DisarmOnExit disarm;
  const u64 n_pad = valid_k(k) ? padded(n, k) : 0;
  if (or_status s = check_transform(agg, n_pad, 4, out, n, sizeof(T), k, base)) return s;
  if (n == 0) return OR_OK;
  if (finalize) {
    if (!count) return OR_ERR_NULL;
    if (ranges_overlap(count, n_pad, out, n * sizeof(T))) return OR_ERR_SHAPE;
  }
  if (masked) {
    if (!stage2_mask) return OR_ERR_NULL;
    if (!aligned(stage2_mask, 4)) return OR_ERR_ALIGN;
    if (ranges_overlap(stage2_mask, n_pad / 8, out, n * sizeof(T))) return OR_ERR_SHAPE;
  }
  const orhost::KernelTable* t = orhost::table_for_class(class_of(k));
  PathArgs a = {};
  a.in = agg; a.count_in = count; a.masks = stage2_mask; a.out = out; a.n = n; a.n_pad = n_pad; a.seed = seed;
  a.base = base; a.k = k;
  a.scale = scale_of(k);
  const u64 units = (n_pad + ((u64)1 << t->tile_log2) - 1) >> t->tile_log2;
  a.unit0 = full_units(n, k, t->tile_log2);
  orhost::launch_fn f = masked     ? (bf16 ? t->decode_masked_bf16 : t->decode_masked_f32)
                        : finalize ? (bf16 ? t->finalize_decode_bf16 : t->finalize_decode_f32)
                                   : (bf16 ? t->decode_bf16 : t->decode_f32);
  return finish(f(a, units, (hipStream_t)stream, orhost::LAUNCH_ONLY));
}

or_status check_reduce(const void* shards, const uint32_t* masks, int N, u64 L, int es) {
  if (N < 1 || N > OR_MAX_WORKERS) return OR_ERR_WORKERS;
  if (L % 32) return OR_ERR_SHAPE;
  if (L > ((u64)1 << 40)) return OR_ERR_SHAPE;
  if (L == 0) return OR_OK;
  if (!shards || !masks) return OR_ERR_NULL;
  if (!aligned(shards, 16) || !aligned(masks, 4)) return OR_ERR_ALIGN;
  if ((L * es) % 16) return OR_ERR_SHAPE;  // every worker's row must start 16-byte aligned
  return OR_OK;
}

template <class T>
or_status masked_reduce_impl(const T* shards, const uint32_t* masks, int N, u64 L, float* sum_out, uint8_t* count_out,
                             void* stream) {
  DisarmOnExit disarm;
  if (or_status s = check_reduce(shards, masks, N, L, sizeof(T))) return s;
  if (L == 0) return OR_OK;
  if (!sum_out || !count_out) return OR_ERR_NULL;
  if (!aligned(sum_out, 16) || !aligned(count_out, 4)) return OR_ERR_ALIGN;
  const u64 in_bytes = (u64)N * L * sizeof(T), mask_bytes = (u64)N * (L / 8);
  if (ranges_overlap(sum_out, L * 4, shards, in_bytes) || ranges_overlap(count_out, L, shards, in_bytes) ||
      ranges_overlap(sum_out, L * 4, masks, mask_bytes) || ranges_overlap(count_out, L, masks, mask_bytes) ||
      ranges_overlap(sum_out, L * 4, count_out, L))
    return OR_ERR_SHAPE;
  constexpr int VEC = 16 / sizeof(T);
  return finish(launch_masked_reduce<T, VEC>(shards, masks, N, L, sum_out, count_out, (hipStream_t)stream,
                                             orhost::LAUNCH_ONLY));
}

size_t workspace_bytes(u64 L, int k) {
  if (!valid_k(k) || k <= 14) return 0;
  const u64 sums = (L * 4 + 255) / 256 * 256;
  const u64 counts = (L + 255) / 256 * 256;
  return (size_t)(sums + counts);
}

// argument checks shared by or_reduce_decode*, or_fused_path* and the batched form (es = element bytes)
or_status check_path(const void* in, const uint32_t* masks, int N, u64 L, int k, u64 base, void* out, uint8_t* count_out,
                     void* ws, size_t ws_bytes, int es) {
  if (!valid_k(k)) return OR_ERR_BLOCK;
  if (or_status s = check_reduce(in, masks, N, L, es)) return s;
  if (L % ((u64)1 << k)) return OR_ERR_SHAPE;
  if (check_base(k, base)) return OR_ERR_SHAPE;
  if (L == 0) return OR_OK;
  if (!out) return OR_ERR_NULL;
  if (!aligned(out, 16)) return OR_ERR_ALIGN;
  const u64 in_bytes = (u64)N * L * es, mask_bytes = (u64)N * (L / 8);
  if (ranges_overlap(out, L * es, in, in_bytes) || ranges_overlap(out, L * es, masks, mask_bytes))
    return OR_ERR_SHAPE;
  if (count_out && (ranges_overlap(count_out, L, in, in_bytes) || ranges_overlap(count_out, L, masks, mask_bytes) ||
                    ranges_overlap(count_out, L, out, L * es)))
    return OR_ERR_SHAPE;
  const size_t need = workspace_bytes(L, k);
  if (need) {
    if (!ws || ws_bytes < need) return OR_ERR_WORKSPACE;
    if (!aligned(ws, 256)) return OR_ERR_ALIGN;
    if (ranges_overlap(ws, need, in, in_bytes) || ranges_overlap(ws, need, masks, mask_bytes) ||
        ranges_overlap(ws, need, out, L * es) || (count_out && ranges_overlap(ws, need, count_out, L)))
      return OR_ERR_SHAPE;
  }
  return OR_OK;
}

// enqueue one checked shard: T = float or uint16_t (bf16 bits).  `allow` = which of this entry point's first /
// last launches this shard may be (timing events ride on those only); `total`, if not null, is expected to be
// zero already and receives the number of arrivals.
template <class T>
or_status run_path(bool fused, const T* in, const uint32_t* masks, int N, u64 L, int k, u64 seed, u64 base, T* out,
                   uint8_t* count_out, void* ws, void* stream, bool bf16, int allow = orhost::LAUNCH_ONLY,
                   unsigned long long* total = nullptr) {
  if (L == 0) return OR_OK;
  const size_t need = workspace_bytes(L, k);
  const orhost::KernelTable* t = orhost::table_for_class(class_of(k));
  hipStream_t s = (hipStream_t)stream;
  const u64 units = (L + ((u64)1 << t->tile_log2) - 1) >> t->tile_log2;
  const int first = orhost::LAUNCH_FIRST & allow, last = orhost::LAUNCH_LAST & allow;
  PathArgs a = {};
  a.in = in; a.masks = masks; a.out = out; a.count_out = count_out; a.n = L; a.n_pad = L; a.seed = seed; a.base = base;
  a.N = N; a.k = k; a.scale = scale_of(k); a.total_out = total;
  if (!need) {
    orhost::launch_fn f = fused ? (bf16 ? t->fused_bf16 : t->fused_f32) : (bf16 ? t->reduce_decode_bf16 : t->reduce_decode_f32);
    return finish(f(a, units, s, first | last));
  }
  // a block spans several tiles: stop at the mean (or sum and count) in the workspace, then decode it
  float* ws_f32 = (float*)ws;
  uint8_t* ws_cnt = (uint8_t*)ws + (L * 4 + 255) / 256 * 256;
  PathArgs d = {};
  d.out = out; d.n = L; d.n_pad = L; d.seed = seed; d.base = base; d.k = k; d.scale = a.scale;
  d.in = ws_f32;
  d.unit0 = units;   // shards hold whole blocks: no tile of the decode needs bounds checks
  if (fused && bf16) {
    // bf16: one kernel does everything.  Workspace: [hand-over slots of the workgroup pairs, 4 L bytes, k = 16 only]
    // [sign stream of the shard, L/8 bytes][pair flags, 8 bytes a block]
    const u64 counters = L >> 7, nflags = k == 16 ? 2 * (L >> 16) : 0;   // one thread per Philox counter
    unsigned* flags = (unsigned*)(ws_cnt + (L / 8 + 255) / 256 * 256);
    const u64 blocks = ((counters > nflags ? counters : nflags) + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return OR_ERR_SHAPE;
    if (hipError_t e = orhost::launch_kernel(k_sign_table, dim3((unsigned)blocks), dim3(256), s, first, (uint4*)ws_cnt, seed,
                                             base >> 7, counters, flags, nflags))
      return finish(e);
    a.sign_tab = (const u64*)ws_cnt;
    a.mean_out = ws_f32;
    a.count_in = (const uint8_t*)flags;
    return finish(t->fused_bf16(a, units, s, last));
  }
  if (fused) {
    // the sign table takes the part of the workspace that the unfused path uses for counts (L/8 of its L bytes)
    const u64 counters = L >> 7;
    if ((counters + 255) / 256 > 0x7FFFFFFFull) return OR_ERR_SHAPE;
    if (hipError_t e = orhost::launch_kernel(k_sign_table, dim3((unsigned)((counters + 255) / 256)), dim3(256), s,
                                             first, (uint4*)ws_cnt, seed, base >> 7, counters, (unsigned*)nullptr, (u64)0))
      return finish(e);
    a.sign_tab = (const u64*)ws_cnt;
    if (k == 15)   // two tiles per block: the fused kernel decodes as well
      return finish(t->fused_f32(a, units, s, last));
    a.mean_out = ws_f32;
    a.out = nullptr;
    if (hipError_t e = t->fused_f32(a, units, s, 0)) return finish(e);
    return finish(t->decode_f32(d, units, s, last));
  }
  uint8_t* cnt = count_out ? count_out : ws_cnt;
  constexpr int VEC = 16 / sizeof(T);
  if (hipError_t e = launch_masked_reduce<T, VEC>(in, masks, N, L, ws_f32, cnt, s, first)) return finish(e);
  d.count_in = cnt;
  if (total) {
    u64 blocks = (L / 16 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (hipError_t e = orhost::launch_kernel(k_received_total, dim3((unsigned)(blocks ? blocks : 1)), dim3(256), s, 0,
                                             (const uint8_t*)cnt, L, total))
      return finish(e);
  }
  return finish((bf16 ? t->finalize_decode_bf16 : t->finalize_decode_f32)(d, units, s, last));
}

template <class T>
or_status path_impl(bool fused, const T* in, const uint32_t* masks, int N, u64 L, int k, u64 seed, u64 base, T* out,
                    uint8_t* count_out, void* ws, size_t ws_bytes, void* stream, bool bf16) {
  DisarmOnExit disarm;
  if (or_status s = check_path(in, masks, N, L, k, base, out, count_out, ws, ws_bytes, sizeof(T))) return s;
  return run_path<T>(fused, in, masks, N, L, k, seed, base, out, count_out, ws, stream, bf16);
}

template <class Out>
or_status finalize_impl(const float* sum, const uint8_t* count, u64 L, Out* mean, void* stream) {
  DisarmOnExit disarm;
  if (L % 32 || L > ((u64)1 << 40)) return OR_ERR_SHAPE;
  if (L == 0) return OR_OK;
  if (!sum || !count || !mean) return OR_ERR_NULL;
  if (!aligned(sum, 16) || !aligned(count, 4) || !aligned(mean, 16)) return OR_ERR_ALIGN;
  if (ranges_overlap(mean, L * sizeof(Out), count, L)) return OR_ERR_SHAPE;
  if (ranges_overlap(mean, L * sizeof(Out), sum, L * 4) && !((const void*)mean == (const void*)sum && sizeof(Out) == 4))
    return OR_ERR_SHAPE;
  const u64 blocks = (L / 4 + 255) / 256;
  if (blocks > 0x7FFFFFFFull) return OR_ERR_SHAPE;
  return finish(orhost::launch_kernel(k_finalize<Out>, dim3((unsigned)blocks), dim3(256), (hipStream_t)stream,
                                      orhost::LAUNCH_ONLY, sum, count, L, mean));
}

or_status received_total_impl(const uint8_t* count, u64 L, unsigned long long* total, void* stream) {
  DisarmOnExit disarm;
  if (L > ((u64)1 << 40)) return OR_ERR_SHAPE;
  if (!total) return OR_ERR_NULL;
  if (!aligned(total, 8)) return OR_ERR_ALIGN;
  if (L && !count) return OR_ERR_NULL;
  if (L && !aligned(count, 16)) return OR_ERR_ALIGN;
  if (L && ranges_overlap(total, 8, count, L)) return OR_ERR_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  if (hipError_t e = orhost::launch_kernel(k_zero_u64, dim3(1), dim3(1), s, L ? orhost::LAUNCH_FIRST : orhost::LAUNCH_ONLY,
                                           total))
    return finish(e);
  if (L == 0) return OR_OK;
  u64 blocks = (L / 16 + 255) / 256;
  if (blocks > 4096) blocks = 4096;   // grid-stride: a few atomics per CU are enough
  if (blocks == 0) blocks = 1;
  return finish(orhost::launch_kernel(k_received_total, dim3((unsigned)blocks), dim3(256), s, orhost::LAUNCH_LAST, count, L,
                                      total));
}

or_status pairs_impl(const float* sums, const uint8_t* counts, const uint32_t* masks, int G, u64 L, float* sum_out,
                     uint8_t* count_out, void* stream) {
  DisarmOnExit disarm;
  if (or_status s = check_reduce(sums, masks, G, L, 4)) return s;
  if (L == 0) return OR_OK;
  if (!counts || !sum_out || !count_out) return OR_ERR_NULL;
  if (!aligned(counts, 4) || !aligned(sum_out, 16) || !aligned(count_out, 4)) return OR_ERR_ALIGN;
  const u64 sb = (u64)G * L * 4, cb = (u64)G * L, mb = (u64)G * (L / 8);
  if (ranges_overlap(sum_out, L * 4, sums, sb) || ranges_overlap(sum_out, L * 4, counts, cb) ||
      ranges_overlap(sum_out, L * 4, masks, mb) || ranges_overlap(count_out, L, sums, sb) ||
      ranges_overlap(count_out, L, counts, cb) || ranges_overlap(count_out, L, masks, mb) ||
      ranges_overlap(sum_out, L * 4, count_out, L))
    return OR_ERR_SHAPE;
  const u64 blocks = (L / 4 + 255) / 256;
  if (blocks > 0x7FFFFFFFull) return OR_ERR_SHAPE;
  return finish(orhost::launch_kernel(k_masked_reduce_pairs, dim3((unsigned)blocks), dim3(256), (hipStream_t)stream,
                                      orhost::LAUNCH_ONLY, sums, counts, masks, G, L, sum_out, count_out));
}

// How the non-empty buckets of a batched call are spread over launches: as few launches as the descriptor
// limit allows, the buckets divided evenly among them.
struct BatchPlan {
  int nonempty, launches, per_launch;
};
BatchPlan plan_batches(int nonempty) {
  BatchPlan p = {nonempty, 0, 0};
  if (nonempty > 0) {
    p.launches = (nonempty + ordev::kMaxBatch - 1) / ordev::kMaxBatch;
    p.per_launch = (nonempty + p.launches - 1) / p.launches;
  }
  return p;
}

// no output of one bucket may touch anything of another bucket (the buckets of a launch run concurrently)
struct Span { const void* p; u64 bytes; bool written; };
template <int NS>
or_status check_disjoint(const Span (&a)[NS], const Span (&b)[NS]) {
  for (int i = 0; i < NS; ++i)
    for (int j = 0; j < NS; ++j)
      if ((a[i].written || b[j].written) && a[i].p && b[j].p && a[i].bytes && b[j].bytes &&
          ranges_overlap(a[i].p, a[i].bytes, b[j].p, b[j].bytes))
        return OR_ERR_SHAPE;
  return OR_OK;
}

hipError_t zero_totals(unsigned long long* totals, int n, hipStream_t s, int pos) {
  return orhost::launch_kernel(k_zero_u64n, dim3((unsigned)((n + 255) / 256)), dim3(256), s, pos, totals, n);
}

// or_fused_path_batched* (fused = true) and or_reduce_decode_batched (fused = false)
or_status path_batched_impl(bool fused, const or_bucket* buckets, int n, int N, int k, bool bf16,
                            unsigned long long* totals, void* ws, size_t ws_bytes, void* stream) {
  DisarmOnExit disarm;
  if (n < 0) return OR_ERR_SHAPE;
  if (n == 0) return OR_OK;
  if (!buckets) return OR_ERR_NULL;
  if (totals && !aligned(totals, 8)) return OR_ERR_ALIGN;
  const u64 es = bf16 ? 2 : 4;
  const Span tot = {totals, totals ? (u64)n * 8 : 0, true};
  // ---- every bucket is checked before anything is enqueued
  int nonempty = 0;
  for (int j = 0; j < n; ++j) {
    const or_bucket& q = buckets[j];
    if (or_status s = check_path(q.grads, q.masks, N, q.shard_len, k, q.base_index, q.out, q.count_out, ws, ws_bytes, (int)es))
      return s;
    if (q.shard_len == 0) continue;
    ++nonempty;
    const u64 L = q.shard_len;
    const Span a[5] = {{q.grads, (u64)N * L * es, false}, {q.masks, (u64)N * (L / 8), false}, {q.out, L * es, true},
                       {q.count_out, L, true}, {ws, workspace_bytes(L, k), true}};
    const Span t5[5] = {tot, {}, {}, {}, {}};
    if (check_disjoint(a, t5)) return OR_ERR_SHAPE;
    for (int i = 0; i < j; ++i) {
      const or_bucket& r = buckets[i];
      const u64 M = r.shard_len;
      const Span b[5] = {{r.grads, (u64)N * M * es, false}, {r.masks, (u64)N * (M / 8), false}, {r.out, M * es, true},
                         {r.count_out, M, true}, {}};
      if (check_disjoint(a, b)) return OR_ERR_SHAPE;
    }
  }
  const orhost::KernelTable* t = orhost::table_for_class(class_of(k));
  orhost::batch_fn f = fused ? (bf16 ? t->fused_batched_bf16 : t->fused_batched_f32)
                             : (bf16 ? t->reduce_decode_batched_bf16 : t->reduce_decode_batched_f32);
  const BatchPlan plan = plan_batches(nonempty);
  hipStream_t s = (hipStream_t)stream;
  // ---- enqueue: the entry point's very first launch carries the start event, its last one the stop event
  bool first_pending = true;
  if (totals) {
    if (hipError_t e = zero_totals(totals, n, s, nonempty ? orhost::LAUNCH_FIRST : orhost::LAUNCH_ONLY)) return finish(e);
    first_pending = false;
  }
  if (!nonempty) return OR_OK;
  int seen = 0;
  if (!f) {   // blocks above 2^14: one bucket after the other, sharing the workspace in stream order
    for (int j = 0; j < n; ++j) {
      const or_bucket& q = buckets[j];
      if (q.shard_len == 0) continue;
      ++seen;
      const int allow = (first_pending ? orhost::LAUNCH_FIRST : 0) | (seen == nonempty ? orhost::LAUNCH_LAST : 0);
      first_pending = false;
      unsigned long long* one = totals ? totals + j : nullptr;
      or_status st = bf16 ? run_path<uint16_t>(fused, (const uint16_t*)q.grads, q.masks, N, q.shard_len, k, q.seed,
                                               q.base_index, (uint16_t*)q.out, q.count_out, ws, stream, true, allow, one)
                          : run_path<float>(fused, (const float*)q.grads, q.masks, N, q.shard_len, k, q.seed, q.base_index,
                                            (float*)q.out, q.count_out, ws, stream, false, allow, one);
      if (st) return st;
    }
    return OR_OK;
  }
  for (int j = 0; seen < nonempty;) {
    ordev::BatchArgs ba = {};
    ba.N = N; ba.k = k; ba.scale = scale_of(k); ba.totals = totals;
    u64 tiles = 0;
    int m = 0;
    for (; j < n && m < plan.per_launch; ++j) {
      const or_bucket& q = buckets[j];
      if (q.shard_len == 0) {
        if (totals && m) { ++j; break; }   // totals[first + m] is bucket first + m: a run of buckets without a gap
        continue;
      }
      const u64 units = (q.shard_len + ((u64)1 << t->tile_log2) - 1) >> t->tile_log2;
      if (tiles + units > 0x7FFFFFFFull) {
        if (m == 0) return OR_ERR_SHAPE;   // cannot happen: check_path bounds the shard length
        break;
      }
      if (m == 0) ba.first = j;
      ba.tile_start[m] = (uint32_t)tiles;
      ba.b[m] = {q.grads, q.masks, q.out, q.count_out, q.shard_len, q.seed, q.base_index};
      tiles += units;
      ++m;
    }
    ba.n = m;
    ba.tile_start[m] = (uint32_t)tiles;
    seen += m;
    const int pos = (first_pending ? orhost::LAUNCH_FIRST : 0) | (seen == nonempty ? orhost::LAUNCH_LAST : 0);
    first_pending = false;
    if (hipError_t e = f(ba, tiles, s, pos)) return finish(e);
  }
  return OR_OK;
}

// one bucket of the separate calls on several buckets
or_status check_stage_bucket(const or_stage_bucket& q, bool reduce, int N, int k, u64 es) {
  const u64 L = q.shard_len;
  if (L % 32 || L > ((u64)1 << 40)) return OR_ERR_SHAPE;
  if (L == 0) return OR_OK;
  if (!q.sum || !q.count) return OR_ERR_NULL;
  if (!aligned(q.sum, 16) || !aligned(q.count, 4)) return OR_ERR_ALIGN;
  if (ranges_overlap(q.sum, L * 4, q.count, L)) return OR_ERR_SHAPE;
  if (reduce) {
    if (or_status s = check_reduce(q.shards, q.masks, N, L, (int)es)) return s;
    const u64 in_bytes = (u64)N * L * es, mask_bytes = (u64)N * (L / 8);
    if (ranges_overlap(q.sum, L * 4, q.shards, in_bytes) || ranges_overlap(q.count, L, q.shards, in_bytes) ||
        ranges_overlap(q.sum, L * 4, q.masks, mask_bytes) || ranges_overlap(q.count, L, q.masks, mask_bytes))
      return OR_ERR_SHAPE;
  } else {
    if (L % ((u64)1 << k)) return OR_ERR_SHAPE;   // buckets hold whole blocks
    if (check_base(k, q.base_index)) return OR_ERR_SHAPE;
    if (!q.out) return OR_ERR_NULL;
    if (!aligned(q.out, 16)) return OR_ERR_ALIGN;
    if (ranges_overlap(q.out, L * es, q.count, L)) return OR_ERR_SHAPE;
    if (ranges_overlap(q.out, L * es, q.sum, L * 4) && !((const void*)q.out == (const void*)q.sum && es == 4))
      return OR_ERR_SHAPE;   // in place is allowed for fp32: a workgroup reads its whole tile before it writes
  }
  return OR_OK;
}

// or_masked_reduce_batched (reduce = true) and or_finalize_decode_batched (reduce = false)
or_status stage_batched_impl(bool reduce, const or_stage_bucket* buckets, int n, int N, int k, bool bf16, void* stream) {
  DisarmOnExit disarm;
  if (n < 0) return OR_ERR_SHAPE;
  if (!reduce && !valid_k(k)) return OR_ERR_BLOCK;
  if (reduce && (N < 1 || N > OR_MAX_WORKERS)) return OR_ERR_WORKERS;
  if (n == 0) return OR_OK;
  if (!buckets) return OR_ERR_NULL;
  const u64 es = bf16 ? 2 : 4;
  int nonempty = 0;
  for (int j = 0; j < n; ++j) {
    const or_stage_bucket& q = buckets[j];
    if (or_status s = check_stage_bucket(q, reduce, N, k, es)) return s;
    if (q.shard_len == 0) continue;
    ++nonempty;
    const u64 L = q.shard_len;
    const Span a[5] = {{reduce ? q.shards : nullptr, (u64)N * L * es, false}, {reduce ? q.masks : nullptr, (u64)N * (L / 8), false},
                       {q.sum, L * 4, reduce}, {q.count, L, reduce}, {reduce ? nullptr : q.out, L * es, true}};
    for (int i = 0; i < j; ++i) {
      const or_stage_bucket& r = buckets[i];
      const u64 M = r.shard_len;
      const Span b[5] = {{reduce ? r.shards : nullptr, (u64)N * M * es, false}, {reduce ? r.masks : nullptr, (u64)N * (M / 8), false},
                         {r.sum, M * 4, reduce}, {r.count, M, reduce}, {reduce ? nullptr : r.out, M * es, true}};
      if (check_disjoint(a, b)) return OR_ERR_SHAPE;
    }
  }
  if (!nonempty) return OR_OK;
  hipStream_t s = (hipStream_t)stream;
  const BatchPlan plan = plan_batches(nonempty);
  const orhost::KernelTable* t = reduce ? nullptr : orhost::table_for_class(class_of(k));
  orhost::batch_fn f = reduce ? nullptr : (bf16 ? t->finalize_decode_batched_bf16 : t->finalize_decode_batched_f32);
  const u64 per_wg = reduce ? 256 * (16 / es) : ((u64)1 << t->tile_log2);   // entries one workgroup serves
  int seen = 0;
  if (!reduce && !f) {   // blocks above 2^14: one bucket after the other
    for (int j = 0; j < n; ++j) {
      const or_stage_bucket& q = buckets[j];
      if (q.shard_len == 0) continue;
      ++seen;
      PathArgs d = {};
      d.in = q.sum; d.count_in = q.count; d.out = q.out; d.n = d.n_pad = q.shard_len; d.seed = q.seed; d.base = q.base_index;
      d.k = k; d.scale = scale_of(k);
      const u64 units = q.shard_len >> t->tile_log2;
      d.unit0 = units;
      const int pos = (seen == 1 ? orhost::LAUNCH_FIRST : 0) | (seen == nonempty ? orhost::LAUNCH_LAST : 0);
      if (hipError_t e = (bf16 ? t->finalize_decode_bf16 : t->finalize_decode_f32)(d, units, s, pos)) return finish(e);
    }
    return OR_OK;
  }
  for (int j = 0; seen < nonempty;) {
    ReduceBatch rb = {};
    ordev::BatchArgs ba = {};
    rb.N = N;
    ba.k = k; ba.scale = scale_of(k);
    u64 wgs = 0;
    int m = 0;
    for (; j < n && m < plan.per_launch; ++j) {
      const or_stage_bucket& q = buckets[j];
      if (q.shard_len == 0) continue;
      const u64 units = (q.shard_len + per_wg - 1) / per_wg;
      if (wgs + units > 0x7FFFFFFFull) {
        if (m == 0) return OR_ERR_SHAPE;   // cannot happen: the shard length is bounded above
        break;
      }
      rb.start[m] = ba.tile_start[m] = (uint32_t)wgs;
      rb.b[m] = {q.shards, q.masks, q.sum, q.count, q.shard_len};
      ba.b[m] = {q.sum, q.count, q.out, nullptr, q.shard_len, q.seed, q.base_index};
      wgs += units;
      ++m;
    }
    rb.n = ba.n = m;
    rb.start[m] = ba.tile_start[m] = (uint32_t)wgs;
    const int pos = (seen == 0 ? orhost::LAUNCH_FIRST : 0) | (seen + m == nonempty ? orhost::LAUNCH_LAST : 0);
    seen += m;
    hipError_t e;
    if (!reduce) e = f(ba, wgs, s, pos);
    else if (bf16) e = orhost::launch_kernel(k_masked_reduce_batched<uint16_t, 8>, dim3((unsigned)wgs), dim3(256), s, pos, rb);
    else e = orhost::launch_kernel(k_masked_reduce_batched<float, 4>, dim3((unsigned)wgs), dim3(256), s, pos, rb);
    if (e) return finish(e);
  }
  return OR_OK;
}

// ------------------------------------------------------------------ scratch for callers that cannot allocate
// or_fused_path_bf16_static: the workspace of the kernels for blocks above 2^14 lives in this array instead of
// caller memory.  Each GPU holds its own copy at its own address; host code never uses the array's name as an
// address, only the pointer that hipGetSymbolAddress returned for the device that is current.
constexpr u64 kStaticMaxShard = OR_STATIC_MAX_SHARD_LEN;
constexpr size_t kScratchBytes = ((kStaticMaxShard * 4 + 255) / 256 * 256) + ((kStaticMaxShard + 255) / 256 * 256);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};

// the scratch array's address on the current device (looked up once per device), or null with *err set
void* scratch_of_current_device(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) {
    *err = hipErrorInvalidDevice;
    return nullptr;
  }
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

// loss > t, exactly: missing / sent is a ratio of integers and t a binary fraction, so both sides are
// compared as integers (no rounded quotient in between)
bool ratio_exceeds(uint64_t missing, uint64_t sent, double t) {
  if (t < 0.0) return true;        // a loss is never negative
  if (t >= 1.0) return false;      // and never above 1
  if (t == 0.0) return missing > 0;
  int e;
  const double fr = frexp(t, &e);                       // t = fr * 2^e, 0.5 <= fr < 1, e <= 0
  const unsigned __int128 mant = (unsigned __int128)(uint64_t)ldexp(fr, 53);   // exact: fr has 53 bits
  const unsigned __int128 prod = mant * sent;           // t * sent = prod / 2^(53 - e); sent < 2^48
  const int sh = 53 - e;                                // >= 53
  if (sh >= 120) return missing > 0;                    // t * sent < 1
  return (unsigned __int128)missing > (prod >> sh);     // missing * 2^sh > prod  <=>  missing > floor(prod / 2^sh)
}

}  // namespace

extern "C" {

uint64_t or_padded_len(uint64_t n, int block_log2) { return valid_k(block_log2) ? padded(n, block_log2) : 0; }
size_t or_workspace_bytes(uint64_t shard_len, int block_log2) { return workspace_bytes(shard_len, block_log2); }
int or_version(void) { return 200; }
int or_last_hip_error(void) { return g_last_hip_error; }

or_status or_time_next_call(void* start_event, void* stop_event) {
  orhost::timing_events() = {(hipEvent_t)start_event, (hipEvent_t)stop_event};
  return OR_OK;
}

const char* or_status_string(or_status s) {
  switch (s) {
    case OR_OK: return "ok";
    case OR_ERR_NULL: return "a required pointer is NULL";
    case OR_ERR_BLOCK: return "block_log2 out of range";
    case OR_ERR_WORKERS: return "worker count out of range";
    case OR_ERR_SHAPE: return "bad length, base_index or overlap";
    case OR_ERR_ALIGN: return "pointer not aligned";
    case OR_ERR_WORKSPACE: return "workspace missing or too small";
    case OR_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

or_status or_rht_encode(const float* grad, uint64_t n, int block_log2, uint64_t seed, float* out, void* stream) {
  return encode_impl<float>(grad, n, block_log2, seed, 0, out, stream, false);
}
or_status or_rht_encode_at(const float* grad, uint64_t n, int block_log2, uint64_t seed, uint64_t base_index,
                           float* out, void* stream) {
  return encode_impl<float>(grad, n, block_log2, seed, base_index, out, stream, false);
}
or_status or_rht_encode_bf16(const uint16_t* grad, uint64_t n, int block_log2, uint64_t seed, uint64_t base_index,
                             uint16_t* out, void* stream) {
  return encode_impl<uint16_t>(grad, n, block_log2, seed, base_index, out, stream, true);
}

or_status or_masked_reduce(const float* shards, const uint32_t* masks, int N, uint64_t shard_len, float* sum_out,
                           uint8_t* count_out, void* stream) {
  return masked_reduce_impl<float>(shards, masks, N, shard_len, sum_out, count_out, stream);
}
or_status or_masked_reduce_bf16(const uint16_t* shards, const uint32_t* masks, int N, uint64_t shard_len,
                                float* sum_out, uint8_t* count_out, void* stream) {
  return masked_reduce_impl<uint16_t>(shards, masks, N, shard_len, sum_out, count_out, stream);
}

or_status or_rht_decode(const float* agg, uint64_t n, int block_log2, uint64_t seed, float* out, void* stream) {
  return decode_impl<float>(agg, nullptr, false, n, block_log2, seed, 0, out, stream, false);
}
or_status or_rht_decode_at(const float* agg, uint64_t n, int block_log2, uint64_t seed, uint64_t base_index,
                           float* out, void* stream) {
  return decode_impl<float>(agg, nullptr, false, n, block_log2, seed, base_index, out, stream, false);
}
or_status or_rht_decode_bf16(const float* agg, uint64_t n, int block_log2, uint64_t seed, uint64_t base_index,
                             uint16_t* out, void* stream) {
  return decode_impl<uint16_t>(agg, nullptr, false, n, block_log2, seed, base_index, out, stream, true);
}

or_status or_finalize_decode(const float* sum, const uint8_t* count, uint64_t n, int block_log2, uint64_t seed,
                             uint64_t base_index, float* out, void* stream) {
  return decode_impl<float>(sum, count, true, n, block_log2, seed, base_index, out, stream, false);
}
or_status or_finalize_decode_bf16(const float* sum, const uint8_t* count, uint64_t n, int block_log2,
                                  uint64_t seed, uint64_t base_index, uint16_t* out, void* stream) {
  return decode_impl<uint16_t>(sum, count, true, n, block_log2, seed, base_index, out, stream, true);
}

or_status or_reduce_decode(const float* shards, const uint32_t* masks, int N, uint64_t shard_len, int block_log2,
                           uint64_t seed, uint64_t base_index, float* out, uint8_t* count_out, void* workspace,
                           size_t workspace_bytes, void* stream) {
  return path_impl<float>(false, shards, masks, N, shard_len, block_log2, seed, base_index, out, count_out, workspace,
                          workspace_bytes, stream, false);
}
or_status or_reduce_decode_bf16(const uint16_t* shards, const uint32_t* masks, int N, uint64_t shard_len,
                                int block_log2, uint64_t seed, uint64_t base_index, uint16_t* out,
                                uint8_t* count_out, void* workspace, size_t workspace_bytes, void* stream) {
  return path_impl<uint16_t>(false, shards, masks, N, shard_len, block_log2, seed, base_index, out, count_out,
                             workspace, workspace_bytes, stream, true);
}
or_status or_fused_path(const float* grads, const uint32_t* masks, int N, uint64_t shard_len, int block_log2,
                        uint64_t seed, uint64_t base_index, float* out, uint8_t* count_out, void* workspace,
                        size_t workspace_bytes, void* stream) {
  return path_impl<float>(true, grads, masks, N, shard_len, block_log2, seed, base_index, out, count_out, workspace,
                          workspace_bytes, stream, false);
}
or_status or_fused_path_bf16(const uint16_t* grads, const uint32_t* masks, int N, uint64_t shard_len,
                             int block_log2, uint64_t seed, uint64_t base_index, uint16_t* out, uint8_t* count_out,
                             void* workspace, size_t workspace_bytes, void* stream) {
  return path_impl<uint16_t>(true, grads, masks, N, shard_len, block_log2, seed, base_index, out, count_out, workspace,
                             workspace_bytes, stream, true);
}

or_status or_fused_path_bf16_static(const uint16_t* grads, const uint32_t* masks, int N, uint64_t shard_len,
                                    int block_log2, uint64_t seed, uint64_t base_index, uint16_t* out,
                                    uint8_t* count_out, void* stream) {
  DisarmOnExit disarm;
  const size_t need = workspace_bytes(shard_len, block_log2);
  if (need && shard_len > kStaticMaxShard) return OR_ERR_WORKSPACE;   // beyond what the static scratch holds
  void* ws = nullptr;
  if (need) {
    hipError_t e;
    ws = scratch_of_current_device(&e);
    if (!ws) return finish(e);
  }
  if (or_status s = check_path(grads, masks, N, shard_len, block_log2, base_index, out, count_out, ws, need, 2)) return s;
  return run_path<uint16_t>(true, grads, masks, N, shard_len, block_log2, seed, base_index, out, count_out, ws, stream, true);
}

or_status or_finalize(const float* sum, const uint8_t* count, uint64_t shard_len, float* mean_out, void* stream) {
  return finalize_impl<float>(sum, count, shard_len, mean_out, stream);
}
or_status or_finalize_bf16(const float* sum, const uint8_t* count, uint64_t shard_len, uint16_t* mean_out,
                           void* stream) {
  return finalize_impl<uint16_t>(sum, count, shard_len, mean_out, stream);
}
or_status or_loss_decision(uint64_t received_total, int N, uint64_t shard_len, const or_loss_policy* policy,
                           int prev_transform_on, int* action_out, int* transform_on_out, double* loss_out) {
  if (!policy || !action_out || !transform_on_out) return OR_ERR_NULL;
  if (N < 1 || N > OR_MAX_WORKERS) return OR_ERR_WORKERS;
  if (policy->transform_on_loss != policy->transform_on_loss || policy->skip_loss != policy->skip_loss ||
      policy->halt_loss != policy->halt_loss)
    return OR_ERR_SHAPE;
  if (shard_len == 0 || shard_len > UINT64_MAX / (uint64_t)N) return OR_ERR_SHAPE;
  const uint64_t sent = (uint64_t)N * shard_len;
  if (received_total > sent) return OR_ERR_SHAPE;
  // the missing arrivals are an exact integer, and every threshold is compared with the exact ratio
  const uint64_t missing = sent - received_total;
  *action_out = ratio_exceeds(missing, sent, policy->halt_loss)
                    ? OR_ACT_HALT
                    : (ratio_exceeds(missing, sent, policy->skip_loss) ? OR_ACT_SKIP : OR_ACT_APPLY);
  *transform_on_out = (prev_transform_on || ratio_exceeds(missing, sent, policy->transform_on_loss)) ? 1 : 0;
  if (loss_out) *loss_out = (double)missing / (double)sent;   // reported value only: one rounding
  return OR_OK;
}

or_status or_received_total(const uint8_t* count, uint64_t shard_len, uint64_t* total_out, void* stream) {
  return received_total_impl(count, shard_len, (unsigned long long*)total_out, stream);
}
or_status or_rht_decode_masked(const float* agg, const uint32_t* mask, uint64_t n, int block_log2, uint64_t seed,
                               uint64_t base_index, float* out, void* stream) {
  return decode_impl<float>(agg, nullptr, false, n, block_log2, seed, base_index, out, stream, false, mask, true);
}
or_status or_rht_decode_masked_bf16(const float* agg, const uint32_t* mask, uint64_t n, int block_log2,
                                    uint64_t seed, uint64_t base_index, uint16_t* out, void* stream) {
  return decode_impl<uint16_t>(agg, nullptr, false, n, block_log2, seed, base_index, out, stream, true, mask, true);
}
or_status or_masked_reduce_pairs(const float* sums, const uint8_t* counts, const uint32_t* masks, int G,
                                 uint64_t shard_len, float* sum_out, uint8_t* count_out, void* stream) {
  return pairs_impl(sums, counts, masks, G, shard_len, sum_out, count_out, stream);
}

or_status or_fused_path_batched(const or_bucket* buckets, int n_buckets, int N, int block_log2, int bf16,
                                void* workspace, size_t workspace_bytes, void* stream) {
  return path_batched_impl(true, buckets, n_buckets, N, block_log2, bf16 != 0, nullptr, workspace, workspace_bytes, stream);
}
or_status or_fused_path_batched_monitored(const or_bucket* buckets, int n_buckets, int N, int block_log2, int bf16,
                                          uint64_t* totals, void* workspace, size_t workspace_bytes, void* stream) {
  return path_batched_impl(true, buckets, n_buckets, N, block_log2, bf16 != 0, (unsigned long long*)totals, workspace,
                           workspace_bytes, stream);
}
or_status or_reduce_decode_batched(const or_bucket* buckets, int n_buckets, int N, int block_log2, int bf16,
                                   uint64_t* totals, void* workspace, size_t workspace_bytes, void* stream) {
  return path_batched_impl(false, buckets, n_buckets, N, block_log2, bf16 != 0, (unsigned long long*)totals, workspace,
                           workspace_bytes, stream);
}
or_status or_masked_reduce_batched(const or_stage_bucket* buckets, int n_buckets, int N, int bf16, void* stream) {
  return stage_batched_impl(true, buckets, n_buckets, N, OR_MIN_LOG2, bf16 != 0, stream);
}
or_status or_finalize_decode_batched(const or_stage_bucket* buckets, int n_buckets, int block_log2, int bf16,
                                     void* stream) {
  return stage_batched_impl(false, buckets, n_buckets, 1, block_log2, bf16 != 0, stream);
}

}  // extern "C"
