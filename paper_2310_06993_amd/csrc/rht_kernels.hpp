// Kernels of the gradient-bucket path (OptiReduce Sec. 3.3 encode/decode, Sec. 3.1.1 aggregation),
// one workgroup per output tile.  See rht_tile.hpp for the tile geometry and the two layouts.
#pragma once
#include "rht_tile.hpp"

namespace ordev {

struct PathArgs {
  const void* in;          // encode: gradient; decode: mean (or sum); reduce/fused: [N][L] shards / raw slices
  const uint8_t* count_in; // finalize+decode: received counts
  const uint32_t* masks;   // [N][L/32]
  void* out;               // result vector
  uint8_t* count_out;      // may be null
  float* mean_out;         // fused without decode: mean in the encoded domain, fp32
  u64 n;                   // valid entries of the input (encode) / output (decode)
  u64 n_pad;               // padded length = vector length on the encoded side; shard_len for reduce/fused
  u64 seed;
  u64 base;                // index of entry 0 in the sign stream
  int N;                   // workers
  int k;                   // block_log2
  float scale;             // 2^(-k/2) rounded to fp32
};

// +1/-1 entry of H_{2^HB}: row `part`, column q
__device__ __forceinline__ float part_coef(int part, int q) { return (__builtin_popcount(part & q) & 1) ? -1.0f : 1.0f; }

template <int K>
__device__ __forceinline__ int tile_bits(int k) { return K ? Geo<K>::KT : k; }

// Signed (and, for blocks above 2^14, +-combined) raw tile of one worker in layout A.
template <int K, class In>
__device__ __forceinline__ void load_signed_tile(const In* __restrict__ x, u64 limit, u64 unit, u64 seed, u64 base,
                                                 int wave, int lane, float (&v)[R], const u64 (&sg_one)[R]) {
  constexpr int T = Geo<K>::T, HB = Geo<K>::HB, PARTS = Geo<K>::PARTS;
  if constexpr (PARTS == 1) {
    load_tile<K, false>(x, unit * T, limit, wave, lane, v);
    apply_signs(v, sg_one);
  } else {
    const u64 blk = unit >> HB;
    const int part = (int)(unit & (PARTS - 1));
#pragma unroll
    for (int r = 0; r < R; ++r) v[r] = 0.0f;
    for (int q = 0; q < PARTS; ++q) {
      const u64 tq = (blk << HB) + q;
      float t[R];
      u64 sg[R];
      load_tile<K, false>(x, tq * T, limit, wave, lane, t);
      sign_masks(seed, base + tq * T + (u64)wave * 1024, sg);
      apply_signs(t, sg);
      const float c = part_coef(part, q);
#pragma unroll
      for (int r = 0; r < R; ++r) v[r] = __builtin_fmaf(c, t[r], v[r]);
    }
  }
}

// Sec. 3.3 encode: out = B^(-1/2) H D x, blockwise; pad of the last block is zero.
template <int K, class In, class Wire>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_encode(PathArgs a) {
  constexpr int T = Geo<K>::T;
  __shared__ float xbuf[Geo<K>::Q > 0 ? T : 1];
  const int wave = wave_id(), lane = lane_id(), kt = tile_bits<K>(a.k);
  const u64 unit = blockIdx.x;
  float v[R];
  u64 sg[R];
  if constexpr (Geo<K>::PARTS == 1) sign_masks(a.seed, a.base + unit * T + (u64)wave * 1024, sg);
  load_signed_tile<K>((const In*)a.in, a.n, unit, a.seed, a.base, wave, lane, v, sg);
  transform_a_to_b<K>(v, xbuf, wave, lane, kt);
  const float c = a.scale * lane_sigma(lane, kt < 6 ? kt : 6);
#pragma unroll
  for (int r = 0; r < R; ++r) v[r] *= c;
  store_tile<K, true>((Wire*)a.out, unit * T, a.n_pad, wave, lane, v);
}

// Mean tile (layout B) for decode: either the mean itself, or sum / count with 0 where count is 0
// (the "averages" of Sec. 3.1.1 taken over the entries that arrived).
template <int K, bool FINALIZE>
__device__ __forceinline__ void load_mean_tile(const PathArgs& a, u64 tile, int wave, int lane, float (&v)[R]) {
  constexpr int T = Geo<K>::T;
  load_tile<K, true>((const float*)a.in, tile * T, a.n_pad, wave, lane, v);
  if constexpr (FINALIZE) {
    float c[R];
    load_tile<K, true>(a.count_in, tile * T, a.n_pad, wave, lane, c);
#pragma unroll
    for (int r = 0; r < R; ++r) v[r] = c[r] > 0.0f ? v[r] / c[r] : 0.0f;
  }
}

// Sec. 3.3 / Sec. 4 decode: out = D B^(-1/2) H mean, first n entries kept.
template <int K, class Out, bool FINALIZE>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_decode(PathArgs a) {
  constexpr int T = Geo<K>::T, HB = Geo<K>::HB, PARTS = Geo<K>::PARTS;
  __shared__ float xbuf[Geo<K>::Q > 0 ? T : 1];
  const int wave = wave_id(), lane = lane_id(), kt = tile_bits<K>(a.k);
  const u64 unit = blockIdx.x;
  float v[R];
  if constexpr (PARTS == 1) {
    load_mean_tile<K, FINALIZE>(a, unit, wave, lane, v);
  } else {
    const u64 blk = unit >> HB;
    const int part = (int)(unit & (PARTS - 1));
#pragma unroll
    for (int r = 0; r < R; ++r) v[r] = 0.0f;
    for (int q = 0; q < PARTS; ++q) {
      float t[R];
      load_mean_tile<K, FINALIZE>(a, (blk << HB) + q, wave, lane, t);
      const float c = part_coef(part, q);
#pragma unroll
      for (int r = 0; r < R; ++r) v[r] = __builtin_fmaf(c, t[r], v[r]);
    }
  }
  transform_b_to_a<K>(v, xbuf, wave, lane, kt);
  const float c = a.scale * lane_sigma(lane, kt < 6 ? kt : 6);
  u64 sg[R];
  sign_masks(a.seed, a.base + unit * T + (u64)wave * 1024, sg);
#pragma unroll
  for (int r = 0; r < R; ++r) v[r] *= c;
  apply_signs(v, sg);
  store_tile<K, false>((Out*)a.out, unit * T, a.n, wave, lane, v);
}

// acc += value where the worker's copy arrived; count of arrivals per entry = full + cnt.
__device__ __forceinline__ void masked_accumulate(const float (&v)[R], const u64 (&m)[R], float (&acc)[R],
                                                  int (&cnt)[R], int& full) {
  u64 all = m[0];
#pragma unroll
  for (int r = 1; r < R; ++r) all &= m[r];
  if (all == ~0ull) {
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] += v[r];
    ++full;
  } else {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const bool got = in_mask(m[r]);
      acc[r] += got ? v[r] : 0.0f;
      cnt[r] += got ? 1 : 0;
    }
  }
}

template <int K>
__device__ __forceinline__ void store_counts(uint8_t* count_out, u64 e0, u64 limit, int wave, int lane,
                                             const int (&cnt)[R], int full) {
  if (!count_out) return;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    u64 e = e0 + off_b<K>(wave, r) + lane;
    if (e < limit) count_out[e] = (uint8_t)(cnt[r] + full);
  }
}

// Aggregation of N encoded shards (Sec. 3.1.1), mean over what arrived, decode (Sec. 3.3).  K <= 14.
template <int K, class Wire, class Out>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_reduce_decode(PathArgs a) {
  constexpr int T = Geo<K>::T;
  static_assert(Geo<K>::PARTS == 1, "blocks above 2^14 go through sum/count in memory");
  __shared__ float xbuf[Geo<K>::Q > 0 ? T : 1];
  const int wave = wave_id(), lane = lane_id(), kt = tile_bits<K>(a.k);
  const u64 unit = blockIdx.x, L = a.n_pad;
  float acc[R];
  int cnt[R], full = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) { acc[r] = 0.0f; cnt[r] = 0; }
  for (int i = 0; i < a.N; ++i) {
    float v[R];
    u64 m[R];
    load_tile<K, true>((const Wire*)a.in + (u64)i * L, unit * T, L, wave, lane, v);
    load_masks<K>(a.masks + (u64)i * (L >> 5), unit * T, L, wave, m);
    masked_accumulate(v, m, acc, cnt, full);
  }
  store_counts<K>(a.count_out, unit * T, L, wave, lane, cnt, full);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int c = cnt[r] + full;
    acc[r] = c ? acc[r] / (float)c : 0.0f;
  }
  transform_b_to_a<K>(acc, xbuf, wave, lane, kt);
  const float c = a.scale * lane_sigma(lane, kt < 6 ? kt : 6);
  u64 sg[R];
  sign_masks(a.seed, a.base + unit * T + (u64)wave * 1024, sg);
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] *= c;
  apply_signs(acc, sg);
  store_tile<K, false>((Out*)a.out, unit * T, L, wave, lane, acc);
}

// The whole path for one shard held by one node: the raw slices of N workers are encoded, the
// encoded entries that arrived are summed and counted, the mean is decoded.  The encoded value is
// rounded to the wire type (identity for fp32) before it is summed, so the result is the one the
// three separate calls give.  DECODE = false (blocks above 2^14) stops at the fp32 mean.
template <int K, class In, bool DECODE>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_fused(PathArgs a) {
  constexpr int T = Geo<K>::T;
  static_assert(DECODE == (Geo<K>::PARTS == 1), "decode in the same kernel only when a block is one tile");
  __shared__ float xbuf[Geo<K>::Q > 0 ? T : 1];
  const int wave = wave_id(), lane = lane_id(), kt = tile_bits<K>(a.k);
  const u64 unit = blockIdx.x, L = a.n_pad;
  const float sigma = lane_sigma(lane, kt < 6 ? kt : 6);
  // a power-of-two scale commutes with rounding to the wire type; any other scale is applied first
  const bool scale_first = sizeof(In) == 2 && (a.k & 1);
  u64 sg[R];
  if constexpr (Geo<K>::PARTS == 1) sign_masks(a.seed, a.base + unit * T + (u64)wave * 1024, sg);
  float acc[R];
  int cnt[R], full = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) { acc[r] = 0.0f; cnt[r] = 0; }
  for (int i = 0; i < a.N; ++i) {
    float v[R];
    u64 m[R];
    load_signed_tile<K>((const In*)a.in + (u64)i * L, L, unit, a.seed, a.base, wave, lane, v, sg);
    transform_a_to_b<K>(v, xbuf, wave, lane, kt);
    if (sizeof(In) == 2) {
      const float pre = scale_first ? a.scale : 1.0f;
#pragma unroll
      for (int r = 0; r < R; ++r) v[r] = round_to<In>(v[r] * pre);
    }
    load_masks<K>(a.masks + (u64)i * (L >> 5), unit * T, L, wave, m);
    masked_accumulate(v, m, acc, cnt, full);
  }
  store_counts<K>(a.count_out, unit * T, L, wave, lane, cnt, full);
  const float post = sigma * (scale_first ? 1.0f : a.scale);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int c = cnt[r] + full;
    acc[r] = c ? acc[r] * post / (float)c : 0.0f;
  }
  if constexpr (DECODE) {
    transform_b_to_a<K>(acc, xbuf, wave, lane, kt);
    const float c = a.scale * sigma;
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] *= c;
    apply_signs(acc, sg);
    store_tile<K, false>((In*)a.out, unit * T, L, wave, lane, acc);
  } else {
    store_tile<K, true>(a.mean_out, unit * T, L, wave, lane, acc);
  }
}

}  // namespace ordev
