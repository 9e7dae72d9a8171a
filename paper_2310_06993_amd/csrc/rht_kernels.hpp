// Kernels of the gradient-bucket path (OptiReduce Sec. 3.3 encode/decode, Sec. 3.1.1 aggregation),
// one workgroup per output tile.  See rht_tile.hpp for the tile geometry and the two layouts.
#pragma once
#include "rht_tile.hpp"

// Which kernels read their inputs with nontemporal loads (each choice measured on MI355X; ENCB / DECB
// are the encode / decode kernels for blocks above 2^14 entries, which came out slower with them).
#ifndef OR_NT_FUSED
#define OR_NT_FUSED true
#endif
#ifndef OR_NT_RDEC
#define OR_NT_RDEC true
#endif
#ifndef OR_NT_PAIRS
#define OR_NT_PAIRS true
#endif
#ifndef OR_NT_ENC
#define OR_NT_ENC true
#endif
#ifndef OR_NT_ENCB
#define OR_NT_ENCB false
#endif
#ifndef OR_NT_DECB
#define OR_NT_DECB false
#endif
#ifndef OR_NT_DEC
#define OR_NT_DEC true
#endif

namespace ordev {

struct PathArgs {
  const void* in;          // encode: gradient; decode: mean (or sum); reduce/fused: [N][L] shards / raw slices
  const uint8_t* count_in; // finalize+decode: received counts
  const uint32_t* masks;   // [N][L/32]
  void* out;               // result vector
  uint8_t* count_out;      // may be null
  float* mean_out;         // fused without decode: mean in the encoded domain, fp32
  const u64* sign_tab;     // fused, blocks above 2^14: sign bits of the shard's entries, 64 per word (see k_fused_pairs)
  unsigned long long* total_out;   // may be null: receives the number of (worker, entry) arrivals (Sec. 3.4 loss monitoring)
  u64 n;                   // valid entries of the input (encode) / output (decode)
  u64 n_pad;               // padded length = vector length on the encoded side; shard_len for reduce/fused
  u64 seed;
  u64 base;                // index of entry 0 in the sign stream
  u64 unit0;               // first output tile served by this launch
  int N;                   // workers
  int k;                   // block_log2
  float scale;             // 2^(-k/2) rounded to fp32
};

// In the shard kernels a tile can be cut short only when blocks are smaller than a tile (class 0).
template <int K> constexpr bool kShardTilesFull = (K != 0);
// LDS buffers for the exchange: two (one barrier per exchange) while they fit several workgroups per CU.
template <int K> constexpr int kXbufs = (Geo<K>::Q == 0) ? 0 : (Geo<K>::T * 4 <= 16384 ? 2 : 1);

// +1/-1 entry of H_{2^HB}: row `part`, column q
__device__ __forceinline__ float part_coef(int part, int q) { return (__builtin_popcount(part & q) & 1) ? -1.0f : 1.0f; }

template <int K>
__device__ __forceinline__ int tile_bits(int k) { return K ? Geo<K>::KT : k; }

// ---- blocks above 2^14: one workgroup per block in encode / decode ----------------------------------
// H_{2^k} = H_{2^(k-14)} (x) H_{2^14}: a workgroup holds the block's PARTS tiles in registers (PARTS*R per
// lane), runs the small factor as add/sub between the tiles and the big one tile by tile.  Every input is
// read once and gets its sign once; one Philox evaluation per wavefront covers its part of all the tiles.

// Sign bits of this wavefront's registers in all PARTS tiles of a block, as two vector registers: lane
// q*16 + r holds the 64-bit lane mask of register r of tile q (lo, hi).  `g` = index, in the padded
// vector, of this wavefront's first entry in tile 0 of the block.
template <int K>
__device__ __forceinline__ void block_sign_words(u64 seed, u64 g, uint32_t& lo, uint32_t& hi) {
  static_assert(Geo<K>::R == 16 && Geo<K>::PARTS <= 4, "lane q*16 + r");
  const int l = lane_id(), q = l >> 4, r = l & 15;
  const u64 ctr = ((g + (u64)q * Geo<K>::T) >> 7) + (u64)(r >> 1);   // a counter covers two registers
  const u32x4 w = philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
  lo = (r & 1) ? w.c : w.a;
  hi = (r & 1) ? w.d : w.b;
}
template <int NR>
__device__ __forceinline__ void apply_block_signs(float (&v)[NR], uint32_t lo, uint32_t hi, int q) {
  asm volatile("" : "+v"(lo), "+v"(hi));   // the lane masks of a tile are formed where the tile is used
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    const u64 m = (u64)(uint32_t)__builtin_amdgcn_readlane((int)lo, q * 16 + r) |
                  ((u64)(uint32_t)__builtin_amdgcn_readlane((int)hi, q * 16 + r) << 32);
    v[r] = in_mask(m) ? -v[r] : v[r];
  }
  __builtin_amdgcn_sched_barrier(0);
}
// the factor H_{PARTS} across the tiles, in place
template <int PARTS, int NR>
__device__ __forceinline__ void across_tiles(float (&v)[PARTS][NR]) {
#pragma unroll
  for (int s = 1; s < PARTS; s <<= 1)
#pragma unroll
    for (int q = 0; q < PARTS; ++q)
      if ((q & s) == 0) {
#pragma unroll
        for (int r = 0; r < NR; ++r) {
          const float x = v[q][r], y = v[q + s][r];
          v[q][r] = x + y;
          v[q + s][r] = x - y;
        }
      }
}

// Sec. 3.3 encode: out = B^(-1/2) H D x, blockwise; pad of the last block is zero.
// FULL = true: every tile of this launch lies wholly inside the input and the output (no bounds checks);
// the host sends the ragged end of a vector to a FULL = false launch of its own, so that the checked
// accesses do not cost the common case registers.
template <int K, class In, class Wire, bool FULL>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_encode(PathArgs a) {
  constexpr int T = Geo<K>::T, R = Geo<K>::R;
  static_assert(Geo<K>::PARTS == 1, "larger blocks use k_encode_block");
  __shared__ float xbuf[Geo<K>::Q > 0 ? T : 1];
  const int wave = wave_id(), lane = lane_id(), kt = tile_bits<K>(a.k);
  const u64 unit = a.unit0 + blockIdx.x;
  float v[R];
  load_tile<K, false, FULL, OR_NT_ENC>((const In*)a.in, unit * T, a.n, wave, lane, v);
  u64 sg[R];
  sign_masks(a.seed, a.base + unit * T + (u64)wave * Geo<K>::WAVE_ENTRIES, sg);
  apply_signs(v, sg);
  transform<K, true>(v, xbuf, wave, lane, kt);
  const float c = a.scale * lane_sigma(lane, kt < 6 ? kt : 6);
#pragma unroll
  for (int r = 0; r < R; ++r) v[r] *= c;
  store_tile<K, true, FULL>((Wire*)a.out, unit * T, a.n_pad, wave, lane, v);
}

// The same for blocks above 2^14: workgroup x encodes block a.unit0 / PARTS + x (a.unit0 counts tiles).
// FULL = false: the block is cut short by the end of the input (its pad reads as zero); the output always
// holds whole blocks.
template <int K, class In, class Wire, bool FULL>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_encode_block(PathArgs a) {
  constexpr int T = Geo<K>::T, R = Geo<K>::R, HB = Geo<K>::HB, PARTS = Geo<K>::PARTS;
  static_assert(PARTS > 1, "blocks above 2^14");
  __shared__ float xbuf[2][T];   // the registers allow one workgroup per CU anyway: alternate, one barrier per exchange
  const int wave = wave_id(), lane = lane_id(), kt = Geo<K>::KT;
  const u64 tile0 = a.unit0 + ((u64)blockIdx.x << HB);
  float v[PARTS][R];
#pragma unroll
  for (int q = 0; q < PARTS; ++q) load_tile<K, false, FULL, OR_NT_ENCB>((const In*)a.in, (tile0 + q) * T, a.n, wave, lane, v[q]);
  uint32_t slo, shi;
  block_sign_words<K>(a.seed, a.base + tile0 * T + (u64)wave * Geo<K>::WAVE_ENTRIES, slo, shi);
#pragma unroll
  for (int q = 0; q < PARTS; ++q) apply_block_signs(v[q], slo, shi, q);
  across_tiles<PARTS, R>(v);
  const float c = a.scale * lane_sigma(lane, 6);
#pragma unroll
  for (int p = 0; p < PARTS; ++p) {
    transform<K, true, false>(v[p], xbuf[p & 1], wave, lane, kt);
#pragma unroll
    for (int r = 0; r < R; ++r) v[p][r] *= c;
    store_tile<K, true, true>((Wire*)a.out, (tile0 + p) * T, a.n_pad, wave, lane, v[p]);
  }
}

// Mean tile (layout B) for decode: either the mean itself, or sum / count with 0 where count is 0
// (the "averages" of Sec. 3.1.1 taken over the entries that arrived).  MASKED: second-stage loss
// (the broadcast of the aggregated shard, Sec. 3.1.1): entries whose bit in a.masks is clear never
// arrived and count as zero.
template <int K, bool FINALIZE, bool FULL, bool MASKED>
__device__ __forceinline__ void load_mean_tile(const PathArgs& a, u64 tile, int wave, int lane,
                                               float (&v)[Geo<K>::R]) {
  constexpr int T = Geo<K>::T, R = Geo<K>::R;
  constexpr bool NT = Geo<K>::PARTS == 1 ? OR_NT_DEC : OR_NT_DECB;
  load_tile<K, true, FULL, NT>((const float*)a.in, tile * T, a.n_pad, wave, lane, v);
  if constexpr (FINALIZE) {
    float c[R];
    load_tile<K, true, FULL, NT>(a.count_in, tile * T, a.n_pad, wave, lane, c);
#pragma unroll
    for (int r = 0; r < R; ++r) v[r] = c[r] > 0.0f ? v[r] * __builtin_amdgcn_rcpf(c[r]) : 0.0f;   // as finalize_mean
  }
  if constexpr (MASKED) {
    const uint32_t w = load_mask_words<K, FULL>(a.masks, tile * T, a.n_pad, mask_word_offset<K>(wave, lane));
    if (!all_arrived(w)) {
#pragma unroll
      for (int r = 0; r < R; ++r) v[r] = in_mask(mask_of_reg(w, r)) ? v[r] : 0.0f;
    }
  }
}

// Sec. 3.3 / Sec. 4 decode: out = D B^(-1/2) H mean, first n entries kept.
template <int K, class Out, bool FINALIZE, bool FULL, bool MASKED = false>
__device__ __forceinline__ void decode_tile(const PathArgs& a, u64 unit) {
  constexpr int T = Geo<K>::T, R = Geo<K>::R;
  static_assert(Geo<K>::PARTS == 1, "larger blocks use k_decode_block");
  __shared__ float xbuf[Geo<K>::Q > 0 ? T : 1];
  const int wave = wave_id(), lane = lane_id(), kt = tile_bits<K>(a.k);
  float v[R];
  load_mean_tile<K, FINALIZE, FULL, MASKED>(a, unit, wave, lane, v);
  transform<K, false>(v, xbuf, wave, lane, kt);
  const float c = a.scale * lane_sigma(lane, kt < 6 ? kt : 6);
  u64 sg[R];
  sign_masks(a.seed, a.base + unit * T + (u64)wave * Geo<K>::WAVE_ENTRIES, sg);
#pragma unroll
  for (int r = 0; r < R; ++r) v[r] *= c;
  apply_signs(v, sg);
  store_tile<K, false, FULL>((Out*)a.out, unit * T, a.n, wave, lane, v);
}
template <int K, class Out, bool FINALIZE, bool FULL, bool MASKED = false>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_decode(PathArgs a) {
  decode_tile<K, Out, FINALIZE, FULL, MASKED>(a, a.unit0 + blockIdx.x);
}

// The same for blocks above 2^14 (see k_encode_block).  The input holds whole blocks; FULL = false: the
// output is cut short inside this block.
template <int K, class Out, bool FINALIZE, bool FULL, bool MASKED = false>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_decode_block(PathArgs a) {
  constexpr int T = Geo<K>::T, R = Geo<K>::R, HB = Geo<K>::HB, PARTS = Geo<K>::PARTS;
  static_assert(PARTS > 1, "blocks above 2^14");
  __shared__ float xbuf[2][T];
  const int wave = wave_id(), lane = lane_id(), kt = Geo<K>::KT;
  const u64 tile0 = a.unit0 + ((u64)blockIdx.x << HB);
  float v[PARTS][R];
#pragma unroll
  for (int q = 0; q < PARTS; ++q) load_mean_tile<K, FINALIZE, true, MASKED>(a, tile0 + q, wave, lane, v[q]);
  uint32_t slo, shi;
  block_sign_words<K>(a.seed, a.base + tile0 * T + (u64)wave * Geo<K>::WAVE_ENTRIES, slo, shi);
  across_tiles<PARTS, R>(v);
  const float c = a.scale * lane_sigma(lane, 6);
#pragma unroll
  for (int p = 0; p < PARTS; ++p) {
    transform<K, false, false>(v[p], xbuf[p & 1], wave, lane, kt);
#pragma unroll
    for (int r = 0; r < R; ++r) v[p][r] *= c;
    apply_block_signs(v[p], slo, shi, p);
    store_tile<K, false, FULL>((Out*)a.out, (tile0 + p) * T, a.n, wave, lane, v[p]);
  }
}

// acc += value where the worker's copy arrived.  Arrivals are counted as `full` (workers whose whole
// tile part arrived) plus a per-register byte in cntp (four registers per word; N <= 255 keeps a byte
// from overflowing).  `words` holds the worker's received bits as loaded by load_mask_words.
template <int NR>
__device__ __forceinline__ void masked_accumulate(const float (&v)[NR], uint32_t words, float (&acc)[NR],
                                                  uint32_t (&cntp)[NR / 4], int& full) {
  if (all_arrived(words)) {
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] += v[r];
    ++full;
  } else {
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const bool got = in_mask(mask_of_reg(words, r));
      acc[r] += got ? v[r] : 0.0f;
      cntp[r >> 2] += got ? (1u << (8 * (r & 3))) : 0u;
    }
  }
}

template <int NR>
__device__ __forceinline__ int count_of(const uint32_t (&cntp)[NR / 4], int full, int r) {
  return (int)((cntp[r >> 2] >> (8 * (r & 3))) & 0xFFu) + full;
}

// Sec. 3.4 loss monitoring: adds this wavefront's number of arrivals (its `full` workers count for all of its
// 64 * NR entries, the rest sit in the packed bytes) to *total with one atomic.
template <int NR>
__device__ __forceinline__ void add_arrivals(unsigned long long* total, const uint32_t (&cntp)[NR / 4], int full) {
  uint32_t mine = 0;
#pragma unroll
  for (int r = 0; r < NR / 4; ++r) mine = __builtin_amdgcn_sad_u8(cntp[r], 0u, mine);
  unsigned long long w = mine;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) w += __shfl_xor(w, o, 64);
  w += (unsigned long long)full * (64u * NR);
  if (lane_id() == 0 && w) atomicAdd(total, w);
}

template <int K, bool FULL>
__device__ __forceinline__ void store_counts(uint8_t* count_out, u64 e0, u64 limit, int wave, int lane,
                                             const uint32_t (&cntp)[Geo<K>::R / 4], int full) {
  constexpr int R = Geo<K>::R;
  if (!count_out) return;
  float c[R];
#pragma unroll
  for (int r = 0; r < R; ++r) c[r] = (float)count_of<R>(cntp, full, r);
  store_tile<K, true, FULL, true>(count_out, e0, limit, wave, lane, c);
  __builtin_amdgcn_sched_barrier(0);
}

// mean over what arrived (0 where nothing arrived), times `post`.  The reciprocal of the count comes
// from v_rcp_f32 (1 ulp), far inside the 1e-6 budget of the path.
template <int NR>
__device__ __forceinline__ void finalize_mean(float (&acc)[NR], const uint32_t (&cntp)[NR / 4], int full, float post) {
  uint32_t any = 0;
#pragma unroll
  for (int r = 0; r < NR / 4; ++r) any |= cntp[r];
  if (__builtin_amdgcn_ballot_w64(any != 0) == 0 && full > 0) {
    const float f = post * __builtin_amdgcn_rcpf((float)full);   // every entry arrived `full` times
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] *= f;
  } else {
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const int c = count_of<NR>(cntp, full, r);
      acc[r] = c ? acc[r] * (post * __builtin_amdgcn_rcpf((float)c)) : 0.0f;
    }
  }
}

// Aggregation of N encoded shards (Sec. 3.1.1), mean over what arrived, decode (Sec. 3.3).  K <= 14.
// The next worker's tile is in flight while the current one is accumulated.
template <int K, class Wire, class Out>
__device__ __forceinline__ void reduce_decode_tile(const PathArgs& a, u64 unit) {
  constexpr int T = Geo<K>::T, R = Geo<K>::R;
  constexpr bool FULL = kShardTilesFull<K>;
  static_assert(Geo<K>::PARTS == 1, "blocks above 2^14 go through sum/count in memory");
  __shared__ float xbuf[Geo<K>::Q > 0 ? T : 1];
  const int wave = wave_id(), lane = lane_id(), kt = tile_bits<K>(a.k);
  const u64 L = a.n_pad, e0 = unit * T;
  const Wire* shards = (const Wire*)a.in;
  float acc[R], va[R], vb[R];
  uint32_t ma, mb = 0, cnt[R / 4];
  int full = 0;
  const int moff = mask_word_offset<K>(wave, lane);
  const u64 mrow = L >> 5;
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.0f;
#pragma unroll
  for (int r = 0; r < R / 4; ++r) cnt[r] = 0;
  load_tile<K, true, FULL, OR_NT_RDEC>(shards, e0, L, wave, lane, va);
  ma = load_mask_words<K, FULL>(a.masks, e0, L, moff);
  for (int i = 0; i < a.N; i += 2) {
    if (i + 1 < a.N) {
      load_tile<K, true, FULL, OR_NT_RDEC>(shards + (u64)(i + 1) * L, e0, L, wave, lane, vb);
      mb = load_mask_words<K, FULL>(a.masks + (u64)(i + 1) * mrow, e0, L, moff);
    }
    masked_accumulate(va, ma, acc, cnt, full);
    if (i + 1 < a.N) {
      if (i + 2 < a.N) {
        load_tile<K, true, FULL, OR_NT_RDEC>(shards + (u64)(i + 2) * L, e0, L, wave, lane, va);
        ma = load_mask_words<K, FULL>(a.masks + (u64)(i + 2) * mrow, e0, L, moff);
      }
      masked_accumulate(vb, mb, acc, cnt, full);
    }
  }
  store_counts<K, FULL>(a.count_out, e0, L, wave, lane, cnt, full);
  if (a.total_out) add_arrivals<R>(a.total_out, cnt, full);
  finalize_mean(acc, cnt, full, 1.0f);
  transform<K, false>(acc, xbuf, wave, lane, kt);
  const float c = a.scale * lane_sigma(lane, kt < 6 ? kt : 6);
  u64 sg[R];
  sign_masks(a.seed, a.base + e0 + (u64)wave * Geo<K>::WAVE_ENTRIES, sg);
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] *= c;
  apply_signs(acc, sg);
  store_tile<K, false, FULL, true>((Out*)a.out, e0, L, wave, lane, acc);
}
template <int K, class Wire, class Out>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_reduce_decode(PathArgs a) {
  reduce_decode_tile<K, Wire, Out>(a, blockIdx.x);
}

// The whole path for one shard held by one node: the raw slices of N workers are encoded, the
// encoded entries that arrived are summed and counted, the mean is decoded.  The encoded value is
// rounded to the wire type (identity for fp32) before it is summed, so the result is the one the
// three separate calls give.  Blocks of up to 2^14 entries (one tile per block).
//
// Per worker: sign flip (layout A), transform to layout B, round, add under the received mask.  Tiles of
// 2, 4, 8 or 16 wavefronts x 16 registers use the transposed transform of rht_tile.hpp, in both directions.
// PREFETCH: a second tile buffer, so that the next worker's tile is in flight during the transform (the
// launcher decides from the size of the grid).  Inputs are read once: nontemporal loads.
template <int K, class In, bool PREFETCH>
__device__ __forceinline__ void fused_tile(const PathArgs& a, u64 unit) {
  constexpr int T = Geo<K>::T, NB = kXbufs<K>, R = Geo<K>::R;
  constexpr bool FULL = kShardTilesFull<K>;
  static_assert(!PREFETCH || R == 16, "a second tile buffer only with 16 entries per lane");
  static_assert(Geo<K>::PARTS == 1, "larger blocks use k_fused_pairs");
  constexpr bool TRANSP = (R == 16 && Geo<K>::Q >= 1);    // transform_transposed, both ways
  constexpr int XF = TRANSP ? tr_floats<K> : T;
  constexpr int NBUF = TRANSP ? 2 : NB;
  __shared__ float xbuf[NBUF ? NBUF : 1][NBUF ? XF : 1];
  const int wave = wave_id(), lane = lane_id(), kt = tile_bits<K>(a.k);
  const u64 L = a.n_pad, e0 = unit * T;
  const In* grads = (const In*)a.in;
  const float sigma = TRANSP ? tr_sigma(lane) : lane_sigma(lane, kt < 6 ? kt : 6);
  // a power-of-two scale commutes with rounding to the wire type; any other scale is applied first
  const bool scale_first = sizeof(In) == 2 && (a.k & 1);
  float acc[R], va[R];
  uint32_t cnt[R / 4];
  int full = 0, flip = 0;
  const int moff = mask_word_offset<K>(wave, lane);
  const u64 mrow = L >> 5;
  // the first worker's tile is requested before the signs are computed, so Philox runs under its latency
  load_tile<K, false, FULL, OR_NT_FUSED>(grads, e0, L, wave, lane, va);
  uint32_t ma = load_mask_words<K, FULL>(a.masks, e0, L, moff);
  u64 sg[R];
  sign_masks(a.seed, a.base + e0 + (u64)wave * Geo<K>::WAVE_ENTRIES, sg);
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.0f;
#pragma unroll
  for (int r = 0; r < R / 4; ++r) cnt[r] = 0;

  auto encode_and_add = [&](float (&v)[R], uint32_t words) {
    apply_signs(v, sg);
    if constexpr (TRANSP) {
      transform_transposed<K>(v, xbuf[flip], xbuf[flip ^ 1], wave, lane);
    } else {
      transform<K, true, NB != 2>(v, xbuf[NB == 2 ? flip : 0], wave, lane, kt);
    }
    flip ^= 1;
    if (sizeof(In) == 2) {
      if (scale_first) {
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = round_to<In>(v[r] * a.scale);
      } else {
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = round_to<In>(v[r]);
      }
    }
    masked_accumulate(v, words, acc, cnt, full);
  };
  if constexpr (PREFETCH) {
    // Two tile buffers: the next worker's tile travels while this one is transformed.  The loads inside
    // the loop are unconditional (the last one or two workers are handled after it), so that the count
    // of loads in flight is the same on every path into a wait and the compiler waits for the older
    // tile only.
    float vb[R];
    uint32_t mb;
    auto request = [&](int i, float (&v)[R], uint32_t& words) {
      load_tile<K, false, FULL, OR_NT_FUSED>(grads + (u64)i * L, e0, L, wave, lane, v);
      words = load_mask_words<K, FULL>(a.masks + (u64)i * mrow, e0, L, moff);
    };
    int i = 0;
    for (; i + 2 < a.N; i += 2) {
      request(i + 1, vb, mb);
      encode_and_add(va, ma);
      request(i + 2, va, ma);
      encode_and_add(vb, mb);
    }
    if (i + 1 < a.N) {
      request(i + 1, vb, mb);
      encode_and_add(va, ma);
      encode_and_add(vb, mb);
    } else {
      encode_and_add(va, ma);
    }
  } else {
    for (int i = 0; i < a.N; ++i) {
      encode_and_add(va, ma);
      if (i + 1 < a.N) {
        load_tile<K, false, FULL, OR_NT_FUSED>(grads + (u64)(i + 1) * L, e0, L, wave, lane, va);
        ma = load_mask_words<K, FULL>(a.masks + (u64)(i + 1) * mrow, e0, L, moff);
      }
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  store_counts<K, FULL>(a.count_out, e0, L, wave, lane, cnt, full);
  if (a.total_out) add_arrivals<R>(a.total_out, cnt, full);
  finalize_mean(acc, cnt, full, sigma * (scale_first ? 1.0f : a.scale));
  __builtin_amdgcn_sched_barrier(0);
  if constexpr (TRANSP) {
    transform_transposed<K>(acc, xbuf[flip], xbuf[flip ^ 1], wave, lane);   // the same code takes layout B to A
  } else {
    transform<K, false, NB != 2>(acc, xbuf[NB == 2 ? flip : 0], wave, lane, kt);
  }
  __builtin_amdgcn_sched_barrier(0);
  const float c = a.scale * sigma;
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] *= c;
  apply_signs(acc, sg);
  store_tile<K, false, FULL, true>((In*)a.out, e0, L, wave, lane, acc);
}

template <int K, class In, bool PREFETCH>
__global__ __launch_bounds__(Geo<K>::THREADS) __attribute__((amdgpu_waves_per_eu(Geo<K>::R == 32 ? 4 : 1)))
void k_fused(PathArgs a) {
  fused_tile<K, In, PREFETCH>(a, blockIdx.x);
}

// ---------------------------------------------------------------------------------------------------
// The fused path for blocks of 2^15 / 2^16 entries (PARTS = 2 / 4 tiles per block).  A workgroup produces
// TWO output tiles of its block, p_lo = h and p_hi = h + PARTS/2, from one reading of the block's input
// tiles: with u_q the signed input tiles and H_{2P} = [[H_P, H_P], [H_P, -H_P]],
//     A = sum_{q <  P/2} H[h][q] u_q,   C = sum_{q >= P/2} H[h][q - P/2] u_q,   p_lo = A + C,  p_hi = A - C,
// so the +-1 combination costs half the sign flips and adds per output of the one-tile-per-workgroup
// form, and the inputs are read PARTS/2 times instead of PARTS times.  With four tiles per block it stops at
// the fp32 mean (layout B) in `mean_out` and k_decode_block finishes; with two it decodes its block itself.
template <int K, class In>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_fused_pairs(PathArgs a) {
  constexpr int T = Geo<K>::T, R = Geo<K>::R, HB = Geo<K>::HB, PARTS = Geo<K>::PARTS, HP = PARTS / 2;
  static_assert(PARTS == 2 || PARTS == 4, "two or four tiles per block");
  // bound by the vector ALUs: the transform with lane bits 2..5 turned into register bits (rht_tile.hpp)
  __shared__ float tbuf[2][tr_floats<K>];   // alternate between the two roles: one barrier per transform
  int flip = 0;
  const int wave = wave_id(), lane = lane_id();
  const u64 L = a.n_pad, nblocks = L >> K;
  // workgroup -> (block, h); the HP workgroups of a block sit on one XCD, next to each other
  u64 blk;
  int h;
  if constexpr (HP == 1) {
    blk = blockIdx.x;
    h = 0;
  } else {
    const u64 x = blockIdx.x, slot = x >> 3;
    h = (int)(slot & (HP - 1));
    blk = ((slot / HP) << 3) + (x & 7);
  }
  if (blk >= nblocks) return;
  const u64 t0 = blk << HB;                      // first tile of the block
  const u64 e_lo = (t0 + h) * T, e_hi = (t0 + h + HP) * T;
  const In* grads = (const In*)a.in;
  const float sigma = tr_sigma(lane);
  const bool scale_first = sizeof(In) == 2 && (a.k & 1);
  const int moff = mask_word_offset<K>(wave, lane);
  const u64 mrow = L >> 5;

  float acc_lo[R], acc_hi[R];
  uint32_t cnt_lo[R / 4], cnt_hi[R / 4];
  int full_lo = 0, full_hi = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) acc_lo[r] = acc_hi[r] = 0.0f;
#pragma unroll
  for (int r = 0; r < R / 4; ++r) cnt_lo[r] = cnt_hi[r] = 0;

  // dst (+)= coef * (signed t), t = input tile q.  The sign bits come from a table that a small kernel
  // wrote before this one (a.sign_tab: bit j of word w = entry 64w + j of the shard): the R words of this
  // wavefront's registers are scalar loads that land in scalar register pairs and serve as lane masks as
  // they are.  Forming them from Philox words held in a vector register instead costs two v_readlane per
  // register and worker -- measured, a fifth of this kernel's vector-ALU time.
  typedef const u64 __attribute__((address_space(4))) * table_ptr;
  auto add_signed = [&](float (&dst)[R], const float (&t)[R], int q, float coef, bool first) {
    table_ptr sg = (table_ptr)(a.sign_tab + ((((t0 + q) * T) + (u64)wave * Geo<K>::WAVE_ENTRIES) >> 6));
    asm volatile("" : "+s"(sg));   // the words of a tile are loaded where the tile is used, not hoisted
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float ts = in_mask(sg[r]) ? -t[r] : t[r];
      dst[r] = first ? coef * ts : __builtin_fmaf(coef, ts, dst[r]);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto finish_tile = [&](float (&v)[R], uint32_t m, float (&acc)[R], uint32_t (&cnt)[R / 4], int& full) {
    transform_transposed<K>(v, tbuf[flip], tbuf[flip ^ 1], wave, lane);
    flip ^= 1;
    if (sizeof(In) == 2) {
      if (scale_first) {
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = round_to<In>(v[r] * a.scale);
      } else {
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = round_to<In>(v[r]);
      }
    }
    masked_accumulate(v, m, acc, cnt, full);
  };

  for (int i = 0; i < a.N; ++i) {
    const In* x = grads + (u64)i * L;
    float A[R], C[R], t[R], w[R];
    // up to three tiles in flight: u_0 -> A, u_1 -> t (four-tile blocks), u_HP -> C
    load_tile<K, false, true, OR_NT_PAIRS>(x, t0 * T, L, wave, lane, A);
    if constexpr (HP == 2) load_tile<K, false, true, OR_NT_PAIRS>(x, (t0 + 1) * T, L, wave, lane, t);
    load_tile<K, false, true, OR_NT_PAIRS>(x, (t0 + HP) * T, L, wave, lane, C);
    const uint32_t m_lo = load_mask_words<K, true>(a.masks + (u64)i * mrow, e_lo, L, moff);
    const uint32_t m_hi = load_mask_words<K, true>(a.masks + (u64)i * mrow, e_hi, L, moff);
    add_signed(A, A, 0, 1.0f, true);
    if constexpr (HP == 2) {
      add_signed(A, t, 1, part_coef(h, 1), false);
      load_tile<K, false, true, OR_NT_PAIRS>(x, (t0 + HP + 1) * T, L, wave, lane, t);
    }
    add_signed(C, C, HP, 1.0f, true);
    if constexpr (HP == 2) add_signed(C, t, HP + 1, part_coef(h, 1), false);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      w[r] = A[r] + C[r];
      C[r] = A[r] - C[r];
    }
    finish_tile(w, m_lo, acc_lo, cnt_lo, full_lo);
    finish_tile(C, m_hi, acc_hi, cnt_hi, full_hi);
  }
  __builtin_amdgcn_sched_barrier(0);
  const float post = sigma * (scale_first ? 1.0f : a.scale);
  if (a.total_out) {
    add_arrivals<R>(a.total_out, cnt_lo, full_lo);
    add_arrivals<R>(a.total_out, cnt_hi, full_hi);
  }
  store_counts<K, true>(a.count_out, e_lo, L, wave, lane, cnt_lo, full_lo);
  finalize_mean(acc_lo, cnt_lo, full_lo, post);
  if constexpr (HP == 2) store_tile<K, true, true>(a.mean_out, e_lo, L, wave, lane, acc_lo);
  store_counts<K, true>(a.count_out, e_hi, L, wave, lane, cnt_hi, full_hi);
  finalize_mean(acc_hi, cnt_hi, full_hi, post);
  if constexpr (HP == 2) {
    store_tile<K, true, true>(a.mean_out, e_hi, L, wave, lane, acc_hi);
  } else {
    // Two tiles per block: this workgroup holds the whole mean of its block and decodes it here (no trip of
    // the mean through memory, no decode launch): the factor across the two tiles, the transform of each
    // (layout B to layout A), scale, signs from the table (whose words are in layout-A order).
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float s = acc_lo[r] + acc_hi[r];
      acc_hi[r] = acc_lo[r] - acc_hi[r];
      acc_lo[r] = s;
    }
    const float c = a.scale * sigma;
    auto decode_tile = [&](float (&v)[R], int q) {
      transform_transposed<K>(v, tbuf[flip], tbuf[flip ^ 1], wave, lane);
      flip ^= 1;
      table_ptr sg = (table_ptr)(a.sign_tab + ((((t0 + q) * T) + (u64)wave * Geo<K>::WAVE_ENTRIES) >> 6));
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float x = v[r] * c;
        v[r] = in_mask(sg[r]) ? -x : x;
      }
      store_tile<K, false, true, true>((In*)a.out, (t0 + q) * T, L, wave, lane, v);
    };
    decode_tile(acc_lo, 0);
    decode_tile(acc_hi, 1);
  }
}

// Several buckets of one launch shape class (same N, block size and type) in ONE launch: small buckets
// (a 25 MiB DDP bucket is only ~100 tiles per shard) cannot fill 256 CUs on their own.  Descriptors ride
// in the kernel arguments; workgroup x serves tile x - tile_start[j] of bucket j.
constexpr int kMaxBatch = 64;   // 64 descriptors keep BatchArgs under the 4 KB of kernel arguments
struct BucketArgs {
  const void* in;          // raw slices / encoded shards; finalize+decode: the fp32 sums
  const void* aux;         // received masks [N][L/32]; finalize+decode: the uint8 counts
  void* out;
  uint8_t* count_out;
  u64 shard_len, seed, base;
};
struct BatchArgs {
  int n, N, k;
  float scale;
  unsigned long long* totals;   // may be null: totals[first + j] receives bucket j's number of arrivals
  int first;
  uint32_t tile_start[kMaxBatch + 1];
  BucketArgs b[kMaxBatch];
};

static_assert(sizeof(BatchArgs) <= 4096, "kernel arguments are limited to 4 KB");

// the bucket that workgroup x serves, as the arguments of a single-bucket call; returns the tile inside it
__device__ __forceinline__ u64 bucket_of(const BatchArgs& ba, PathArgs& a) {
  const uint32_t x = blockIdx.x;
  int j = 0;
  while (j + 1 < ba.n && ba.tile_start[j + 1] <= x) ++j;
  a = PathArgs{};
  a.in = ba.b[j].in; a.masks = (const uint32_t*)ba.b[j].aux; a.count_in = (const uint8_t*)ba.b[j].aux;
  a.out = ba.b[j].out; a.count_out = ba.b[j].count_out;
  a.n = a.n_pad = ba.b[j].shard_len; a.seed = ba.b[j].seed; a.base = ba.b[j].base;
  a.N = ba.N; a.k = ba.k; a.scale = ba.scale;
  a.total_out = ba.totals ? ba.totals + ba.first + j : nullptr;
  return x - ba.tile_start[j];
}

template <int K, class In, bool PREFETCH>
__global__ __launch_bounds__(Geo<K>::THREADS) __attribute__((amdgpu_waves_per_eu(Geo<K>::R == 32 ? 4 : 1)))
void k_fused_batched(BatchArgs ba) {
  PathArgs a;
  const u64 unit = bucket_of(ba, a);
  fused_tile<K, In, PREFETCH>(a, unit);
}

// The three-call path on several buckets: aggregation + mean + decode of encoded shards, and mean + decode of
// (sum, count) pairs; every bucket holds whole blocks.
template <int K, class Wire>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_reduce_decode_batched(BatchArgs ba) {
  PathArgs a;
  const u64 unit = bucket_of(ba, a);
  reduce_decode_tile<K, Wire, Wire>(a, unit);
}
template <int K, class Out>
__global__ __launch_bounds__(Geo<K>::THREADS) void k_finalize_decode_batched(BatchArgs ba) {
  PathArgs a;
  const u64 unit = bucket_of(ba, a);
  decode_tile<K, Out, true, kShardTilesFull<K>, false>(a, unit);
}

}  // namespace ordev
