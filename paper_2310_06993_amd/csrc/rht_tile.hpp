// Device-side building blocks for the blockwise randomized Hadamard transform
// (OptiReduce, Sec. 3.3 "Dispersing Gradient Loss") on gfx950.
//
// Work is cut into TILES of 2^TL consecutive entries (TL = max(10, min(k, 14))).
// A tile is owned by one workgroup of W = 2^(TL-10) wavefronts; every lane holds
// 16 entries in registers.  In both register layouts used here a register of a
// wavefront covers 64 CONSECUTIVE entries (lane l <-> entry l of that run), so
//   * every global load/store instruction of a wavefront is one 256-byte run,
//   * the 64 sign bits / 64 received bits of a register are two consecutive
//     32-bit words and live in a scalar register pair used directly as a lane
//     mask (no per-lane bit extraction).
//
// Layout A ("load" layout):  entry = wave*1024 + reg*64 + lane
// Layout B ("wire" layout):  entry = (reg >> RLO)*1024 + ((wave << RLO) + (reg & (2^RLO-1)))*64 + lane
// with RLO = 4 - log2(W).  A and B differ by one exchange through LDS that swaps
// the wave bits with the top register bits; for W = 1 they are the same layout.
//
// Butterfly stages (the Hadamard factors commute, so any order is the same map):
//   entry bits 0..5   : across lanes (DPP / ds_swizzle / ds_bpermute)
//   register bits     : plain add/sub between registers
//   wave bits         : become register bits after the LDS exchange
//
// Lane stages use v <- v + s*neighbour with s = +1 on the lower lane of a pair and
// -1 on the upper one, which leaves the *negated* difference on the upper lane.
// All later stages combine values that sit on the same lane, so the result of a
// whole transform is H x multiplied, on lane l, by parity(l & lane-stage bits).
// That per-lane factor ("sigma") is folded into the scale multiply that follows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ordev {

typedef unsigned long long u64;
typedef const uint32_t __attribute__((address_space(4)))* const_u32_ptr;

constexpr int R = 16;  // entries per lane per tile

// Geometry for a block of 2^K entries.  KT bits are transformed inside a tile; for
// K > 14 the remaining HB bits are handled by combining 2^HB input tiles with +-1
// before the in-tile transform (H_{2^K} = H_{2^HB} (x) H_{2^14}).
// K == 0 stands for "any block_log2 <= 10, taken at run time" (one wavefront per tile).
template <int K>
struct Geo {
  static constexpr int KT = (K == 0) ? 10 : (K > 14 ? 14 : K);
  static constexpr int TL = KT;
  static constexpr int T = 1 << TL;
  static constexpr int Q = TL - 10;
  static constexpr int W = 1 << Q;
  static constexpr int THREADS = 64 * W;
  static constexpr int HB = (K > 14) ? K - 14 : 0;
  static constexpr int PARTS = 1 << HB;
  static constexpr int RLO = 4 - Q;
};

__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

template <int K>
__device__ __forceinline__ int off_a(int wave, int reg) { return wave * 1024 + reg * 64; }
template <int K>
__device__ __forceinline__ int off_b(int wave, int reg) {
  constexpr int RLO = Geo<K>::RLO;
  return (reg >> RLO) * 1024 + (((wave << RLO) + (reg & ((1 << RLO) - 1))) * 64);
}

// ------------------------------------------------------------------ element types
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __builtin_bit_cast(float, (uint32_t)v.bits << 16); }
__device__ __forceinline__ float to_f32(uint8_t v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) {  // round to nearest even
  return bf16_t{__builtin_bit_cast(uint16_t, (__bf16)v)};
}
template <class T> __device__ __forceinline__ float round_to(float v) { return to_f32(from_f32<T>(v)); }

// ------------------------------------------------------------------ Philox4x32-10 (Salmon et al., SC'11)
struct u32x4 { uint32_t a, b, c, d; };
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
#pragma unroll
  for (int i = 0; i < 10; ++i) {
    uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return u32x4{c0, c1, c2, c3};
}

// Sign lane-masks for the 16 registers of this wavefront in layout A.  `g` is the index,
// in the padded vector, of the wavefront's first entry (a multiple of 128).  Entry i flips
// sign iff bit (i mod 128) of Philox(counter = i div 128, key = seed) is set.  Lanes 0..7 each
// produce the 128 bits of one counter; the words move to scalar registers with readlane.
__device__ __forceinline__ void sign_masks(u64 seed, u64 g, u64 (&sg)[R]) {
  u64 ctr = (g >> 7) + (u64)lane_id();
  u32x4 w = philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
#pragma unroll
  for (int r = 0; r < R; ++r) {
    uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)((r & 1) ? w.c : w.a), r >> 1);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)((r & 1) ? w.d : w.b), r >> 1);
    sg[r] = (u64)lo | ((u64)hi << 32);
  }
}

__device__ __forceinline__ bool in_mask(u64 m) { return __builtin_amdgcn_inverse_ballot_w64(m); }

__device__ __forceinline__ void apply_signs(float (&v)[R], const u64 (&sg)[R]) {
#pragma unroll
  for (int r = 0; r < R; ++r) v[r] = in_mask(sg[r]) ? -v[r] : v[r];
}

// ------------------------------------------------------------------ butterflies
template <int BIT>
__device__ __forceinline__ float lane_partner(float v, int xor32_addr) {
  int i = __builtin_bit_cast(int, v);
  int p;
  if constexpr (BIT == 0) p = __builtin_amdgcn_update_dpp(0, i, 0xB1, 0xF, 0xF, true);        // quad_perm [1,0,3,2]
  else if constexpr (BIT == 1) p = __builtin_amdgcn_update_dpp(0, i, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
  else if constexpr (BIT == 2) p = __builtin_amdgcn_ds_swizzle(i, 0x101F);                    // lane ^ 4
  else if constexpr (BIT == 3) p = __builtin_amdgcn_update_dpp(0, i, 0x128, 0xF, 0xF, true);  // row_ror:8 = lane ^ 8
  else if constexpr (BIT == 4) p = __builtin_amdgcn_ds_swizzle(i, 0x401F);                    // lane ^ 16
  else p = __builtin_amdgcn_ds_bpermute(xor32_addr, i);                                       // lane ^ 32
  return __builtin_bit_cast(float, p);
}

template <int BIT>
__device__ __forceinline__ void lane_stage(float (&v)[R], int lane) {
  const float s = (lane >> BIT) & 1 ? -1.0f : 1.0f;
  const int a32 = (lane ^ 32) << 2;
#pragma unroll
  for (int r = 0; r < R; ++r) v[r] = __builtin_fmaf(lane_partner<BIT>(v[r], a32), s, v[r]);
}

// all lane stages for entry bits 0..nbits-1 (nbits uniform, <= 6)
__device__ __forceinline__ void lane_stages(float (&v)[R], int lane, int nbits) {
  if (nbits > 0) lane_stage<0>(v, lane);
  if (nbits > 1) lane_stage<1>(v, lane);
  if (nbits > 2) lane_stage<2>(v, lane);
  if (nbits > 3) lane_stage<3>(v, lane);
  if (nbits > 4) lane_stage<4>(v, lane);
  if (nbits > 5) lane_stage<5>(v, lane);
}

// +1 / -1 factor left on this lane by `nbits` lane stages
__device__ __forceinline__ float lane_sigma(int lane, int nbits) {
  return (__builtin_popcount(lane & ((1 << nbits) - 1)) & 1) ? -1.0f : 1.0f;
}

template <int RBIT>
__device__ __forceinline__ void reg_stage(float (&v)[R]) {
  constexpr int S = 1 << RBIT;
#pragma unroll
  for (int r = 0; r < R; ++r)
    if ((r & S) == 0) {
      float a = v[r], b = v[r + S];
      v[r] = a + b;
      v[r + S] = a - b;
    }
}

// register stages for register-index bits lo..hi-1 (uniform run-time range inside 0..4)
__device__ __forceinline__ void reg_stages(float (&v)[R], int lo, int hi) {
  if (lo <= 0 && hi > 0) reg_stage<0>(v);
  if (lo <= 1 && hi > 1) reg_stage<1>(v);
  if (lo <= 2 && hi > 2) reg_stage<2>(v);
  if (lo <= 3 && hi > 3) reg_stage<3>(v);
}

// LDS exchange between the two layouts (W > 1 only).  xbuf holds one tile of floats, indexed in
// layout-B order: slot = (wave_b*16 + reg_b)*64 + lane.
template <int K, bool A_TO_B>
__device__ __forceinline__ void exchange(float (&v)[R], float* xbuf, int wave, int lane) {
  constexpr int Q = Geo<K>::Q, RLO = Geo<K>::RLO;
  static_assert(Q > 0, "exchange needs more than one wavefront");
  __syncthreads();  // previous readers of xbuf are done
#pragma unroll
  for (int r = 0; r < R; ++r) {
    // layout A register r of wave `wave` is layout B register ((wave << RLO) | r_lo) of wave (r >> RLO)
    int slot_cross = (((r >> RLO) * 16) + ((wave << RLO) | (r & ((1 << RLO) - 1)))) * 64 + lane;
    int slot_own = (wave * 16 + r) * 64 + lane;
    if (A_TO_B) xbuf[slot_cross] = v[r]; else xbuf[slot_own] = v[r];
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    int slot_cross = (((r >> RLO) * 16) + ((wave << RLO) | (r & ((1 << RLO) - 1)))) * 64 + lane;
    int slot_own = (wave * 16 + r) * 64 + lane;
    v[r] = A_TO_B ? xbuf[slot_own] : xbuf[slot_cross];
  }
}

// Unscaled Hadamard transform of one tile over its low `kt` entry bits, layout A in, layout B out.
// Result on lane l carries the factor lane_sigma(l, min(kt, 6)).
template <int K>
__device__ __forceinline__ void transform_a_to_b(float (&v)[R], float* xbuf, int wave, int lane, int kt) {
  constexpr int Q = Geo<K>::Q;
  lane_stages(v, lane, kt < 6 ? kt : 6);
  reg_stages(v, 0, kt <= 6 ? 0 : (kt < 10 ? kt - 6 : 4));
  if constexpr (Q > 0) {
    exchange<K, true>(v, xbuf, wave, lane);
    reg_stages(v, 4 - Q, 4);
  }
}

// Same map, layout B in, layout A out.
template <int K>
__device__ __forceinline__ void transform_b_to_a(float (&v)[R], float* xbuf, int wave, int lane, int kt) {
  constexpr int Q = Geo<K>::Q;
  lane_stages(v, lane, kt < 6 ? kt : 6);
  reg_stages(v, 0, kt <= 6 ? 0 : (kt < 10 ? kt - 6 : 4));
  if constexpr (Q > 0) {
    exchange<K, false>(v, xbuf, wave, lane);
    reg_stages(v, 4 - Q, 4);
  }
}

// ------------------------------------------------------------------ tile loads / stores
// `p` points at entry 0 of the vector, `e0` is the tile's first entry, `limit` the number of valid
// entries of the vector; entries at or beyond `limit` read as zero / are not written.
template <int K, bool LAYOUT_B, class T>
__device__ __forceinline__ void load_tile(const T* __restrict__ p, u64 e0, u64 limit, int wave, int lane,
                                          float (&v)[R]) {
  if (e0 + Geo<K>::T <= limit) {
#pragma unroll
    for (int r = 0; r < R; ++r) v[r] = to_f32(p[e0 + (LAYOUT_B ? off_b<K>(wave, r) : off_a<K>(wave, r)) + lane]);
  } else {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      u64 e = e0 + (LAYOUT_B ? off_b<K>(wave, r) : off_a<K>(wave, r)) + lane;
      v[r] = e < limit ? to_f32(p[e]) : 0.0f;
    }
  }
}

template <int K, bool LAYOUT_B, class T>
__device__ __forceinline__ void store_tile(T* __restrict__ p, u64 e0, u64 limit, int wave, int lane,
                                           const float (&v)[R]) {
  if (e0 + Geo<K>::T <= limit) {
#pragma unroll
    for (int r = 0; r < R; ++r) p[e0 + (LAYOUT_B ? off_b<K>(wave, r) : off_a<K>(wave, r)) + lane] = from_f32<T>(v[r]);
  } else {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      u64 e = e0 + (LAYOUT_B ? off_b<K>(wave, r) : off_a<K>(wave, r)) + lane;
      if (e < limit) p[e] = from_f32<T>(v[r]);
    }
  }
}

// Received-bit lane masks of one worker for this wavefront's 16 registers in layout B.
// `row` = that worker's mask row (bit j of word w = entry 32w+j), `e0` = tile's first entry,
// `limit` = shard length (multiple of 32).  Words wholly beyond `limit` read as 0.
template <int K>
__device__ __forceinline__ void load_masks(const uint32_t* row, u64 e0, u64 limit, int wave, u64 (&m)[R]) {
  const_u32_ptr mp = (const_u32_ptr)(uintptr_t)row;
  if (e0 + Geo<K>::T <= limit) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      u64 w = (e0 + off_b<K>(wave, r)) >> 5;
      m[r] = (u64)mp[w] | ((u64)mp[w + 1] << 32);
    }
  } else {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      u64 e = e0 + off_b<K>(wave, r);
      u64 w = e >> 5;
      uint32_t lo = (e < limit) ? mp[w] : 0u;
      uint32_t hi = (e + 32 < limit) ? mp[w + 1] : 0u;
      m[r] = (u64)lo | ((u64)hi << 32);
    }
  }
}

}  // namespace ordev
