// The fused path (OptiReduce Sec. 3.3 encode, Sec. 3.1.1 aggregation, Sec. 3.3 / Sec. 4 decode) for bf16
// gradients in blocks of 2^15 / 2^16 entries (PARTS = 2 / 4 tiles of 2^14), with the FIRST Hadamard factor of
// the encode on the matrix cores.
//
// The raw input is bf16 and the Hadamard matrix is +-1, so a bf16 product with fp32 accumulation applies a
// factor H_32 exactly.  One v_mfma_f32_16x16x32_bf16 takes, as its B operand, 512 raw entries the way they
// come from memory -- lane l holds 8 consecutive entries (one 16-byte load), lanes 16g .. 16g+15 read from
// "group" g -- and contracts the 3 index bits inside a lane's load and the 2 bits of the group:
//     2^16 blocks: group = input tile q (index bits 14, 15); the workgroup with half index h keeps the 16 rows
//                  with output bit 14 = h, so its outputs are the tiles h and h + 2 (as in k_fused_pairs);
//     2^15 blocks: group = (tile, index bit 9); two products (output bit 9 = 0 / 1) keep all 32 rows.
// That replaces unpacking, the +-1 combination of the tiles and three butterfly stages of the vector form.
// The random signs are applied first, by XOR on the packed pairs: a lane's 8 sign bits are one byte of the
// sign stream (held in registers for the whole block: the signs are the same for every worker), expanded to a
// mask with bit 15 / 31 set by one multiply and one AND per pair.
//
// Positions.  A product leaves D[i][n] on lane l = (n, i2, i3), register i0 i1, with n = l & 15 the untouched index
// bits 3..6.  With the chunk number ch (index bits 7.. of the wavefront's slice) the 32 registers of a lane are two
// arrays X, Y of 16: register 4 ch' + r.  The remaining stages (transform_dpp_sel) swap the bits held by the register
// number with those held by the wave number, as transform_transposed does, and skip the bits the product has done:
//     after the encode   array a, wave w, register r, lane l   is encoded entry
//         y = r*1024 + a*512 + (w>>2)*128 + ((l>>2)&3)*32 + (l&3)*8 + ((l>>4)&1)*4 + (w&3)
//         of the output tile chosen by lane bit 5 (2^16: tiles h, h+2; 2^15: tiles 0, 1);
//     after the decode   array a, wave w, register r, lane l   is decoded entry
//         x = w*1024 + a*512 + (r>>2)*128 + ((l>>2)&3)*32 + (l&3)*8 + ((l>>4)&1)*4 + (r&3)
//         of the tile chosen by lane bit 5 (and, for 2^16, by sum / difference of the two workgroups' results).
// The decode is the plain vector transform of the fp32 mean over all these bits; for 2^16 blocks the last
// factor (index bit 14) joins the two workgroups of a block: the one that finishes first leaves its result in the
// workspace, the other one adds and subtracts and stores all four tiles.
#pragma once
#include "rht_kernels.hpp"

namespace ordev {

typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
typedef float f32x4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {   // round to nearest even, lo in bits 0..15
  typedef float f2 __attribute__((ext_vector_type(2)));
  typedef __bf16 b2 __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{lo, hi}, b2));
}
__device__ __forceinline__ float bf16_lo(uint32_t p) { return __builtin_bit_cast(float, p << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t p) { return __builtin_bit_cast(float, p & 0xFFFF0000u); }

// Scratch of the pair hand-over (four tiles per block), one pair of words per block; zeroed before the kernel.
struct PairFlags {
  unsigned arrived;   // how many of the block's two workgroups have finished their workers
  unsigned ready;     // set by the first one once its result is in the workspace
};
constexpr unsigned kPairSpinLimit = 1u << 22;   // polls of `ready` before the waiting workgroup gives up

// The stages that are left after the matrix-core product: the register bits in FIRST, the lane bits 0..3 as DPP
// stages, the wave bits after the plain exchange between wavefronts (register and wave bits swap, lanes stay in
// place: the same final positions as transform_transposed).  Measured against the form with the transposition inside
// the wavefront (lane bits 2, 3 as register stages): half the LDS traffic for 64 more half-rate vector instructions,
// 6 % less time -- a trip's vector, LDS and memory phases hardly overlap (one workgroup per CU, its wavefronts in step).
// The result on lane l carries the factor lane_sigma(l, 4).
template <int K, int FIRST>
__device__ __forceinline__ void transform_dpp_sel(float (&v)[16], float* xbuf, int wave, int lane) {
  static_assert(Geo<K>::R == 16 && Geo<K>::Q == 4, "16 wavefronts of 16 registers");
  if constexpr (FIRST & 1) reg_stage<0>(v);
  if constexpr (FIRST & 2) reg_stage<1>(v);
  if constexpr (FIRST & 4) reg_stage<2>(v);
  if constexpr (FIRST & 8) reg_stage<3>(v);
  lane_stage<0>(v, lane);
  lane_stage<1>(v, lane);
  lane_stage<2>(v, lane);
  lane_stage<3>(v, lane);
  exchange<K, true, false>(v, xbuf, wave, lane);
  reg_stages(v, 0, 4);
}

// (sign bit of the even entry) << 15 | (sign bit of the odd entry) << 31 for pair d = 0..3 of a lane's 8 entries,
// from their sign byte: the two shifted copies of the byte do not overlap, so the multiply carries nothing
template <int D>
__device__ __forceinline__ uint32_t pair_sign_mask(uint32_t byte) {
  return (byte * ((1u << (15 - 2 * D)) + (1u << (30 - 2 * D)))) & 0x80008000u;
}

template <int K>
__global__ __launch_bounds__(1024) void k_fused_mx(PathArgs a) {
  constexpr int T = Geo<K>::T, R = 16, HB = Geo<K>::HB, PARTS = Geo<K>::PARTS, HP = PARTS / 2;
  constexpr int NCH = HP == 2 ? 8 : 4;            // 16-byte loads of a lane per worker
  static_assert(Geo<K>::R == 16 && Geo<K>::W == 16 && (PARTS == 2 || PARTS == 4), "2^14 tiles, two or four per block");
  __shared__ float tbuf[2][tr_floats<K>];
  __shared__ uint32_t s_clean[16];
  __shared__ unsigned s_order;
  int flip = 0;
  const int wave = wave_id(), lane = lane_id();
  const int nn = lane & 15, grp = lane >> 4, sel = lane >> 5;    // sel: which of the two output tiles this lane holds
  const u64 L = a.n_pad, nblocks = L >> K;
  u64 blk;
  int h;
  if constexpr (HP == 1) {
    blk = blockIdx.x;
    h = 0;
  } else {   // the HP workgroups of a block sit on one XCD (blockIdx modulo 8), next to each other
    const u64 x = blockIdx.x, slot = x >> 3;
    h = (int)(slot & (HP - 1));
    blk = ((slot / HP) << 3) + (x & 7);
  }
  if (blk >= nblocks) return;
  const u64 t0 = blk << HB;
  const u64 e_lo = (t0 + h) * T, e_hi = (t0 + h + HP) * T;       // the two output tiles (lane bit 5 = 0 / 1)
  const bf16_t* grads = (const bf16_t*)a.in;
  const float sigma = tr_sigma(lane);
  constexpr bool scale_first = (K & 1);   // 2^(-k/2) is a power of two for even k and commutes with the rounding
  const u64 mrow = L >> 5;
  const uint8_t* sign_bytes = (const uint8_t*)a.sign_tab;        // bit j of byte b = sign of entry 8 b + j of the shard

  // ---- the +-1 operand(s): lane l holds row i = l & 15, columns 8 (l >> 4) + 0..7
  // column bits 0..2 pair with row bits 0..2; the two group bits pair with (2^16) output bit 14 = h and row bit 3,
  // (2^15) row bit 3 and the product number m
  bf16x8v hmat[HP == 2 ? 1 : 2];
  {
    const int i = lane & 15;
#pragma unroll
    for (int m = 0; m < (HP == 2 ? 1 : 2); ++m) {
      u32x4v w;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        uint32_t pair = 0;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int jj = 2 * d + e;
          int par = __builtin_popcount((i & 7) & jj);
          if constexpr (HP == 2) par += h * (grp & 1) + (i >> 3) * (grp >> 1);
          else par += (i >> 3) * (grp & 1) + m * (grp >> 1);
          pair |= ((par & 1) ? 0xBF80u : 0x3F80u) << (16 * e);
        }
        w[d] = pair;
      }
      hmat[m] = __builtin_bit_cast(bf16x8v, w);
    }
  }
  // ---- where this lane's loads sit: a uniform entry (the wavefront's slice of the block's first tile) plus a
  // 32-bit lane part, so that addresses are a scalar base and one vector register
  const u64 wave_entry = t0 * T + (u64)wave * 1024;
  unsigned lane_part;   // entries from wave_entry to the lane's load of chunk 0
  if constexpr (HP == 2) lane_part = (unsigned)grp * T + nn * 8;
  else lane_part = (unsigned)(grp & 1) * T + (grp >> 1) * 512 + nn * 8;
  // ---- sign bytes of the lane's loads (chunk ch: 8 entries from lane_part + 128 ch), the same for every worker
  uint32_t sbytes[NCH / 4];
  {
    const uint8_t* sb = sign_bytes + (wave_entry >> 3) + (lane_part >> 3);
#pragma unroll
    for (int q = 0; q < NCH / 4; ++q)
      sbytes[q] = (uint32_t)sb[(4 * q) * 16] | ((uint32_t)sb[(4 * q + 1) * 16] << 8) | ((uint32_t)sb[(4 * q + 2) * 16] << 16) |
                  ((uint32_t)sb[(4 * q + 3) * 16] << 24);
  }

  float accX[R], accY[R];
#pragma unroll
  for (int r = 0; r < R; ++r) accX[r] = accY[r] = 0.0f;

  u32x4v p[NCH];
  uint32_t mw;
  // Loads go through buffer descriptors built per worker in scalar registers: one vector register (the lane's byte
  // offset) then serves every load of every worker, where flat addresses would take a 64-bit pair per stream.
  const int lane_bytes = (int)lane_part * 2;
  auto request = [&](int i, int ch0, int ch1) {
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc((void*)(grads + (u64)i * L + wave_entry), 0, PARTS * T * 2, 0x00020000);
#pragma unroll
    for (int ch = ch0; ch < ch1; ++ch)   // four tiles per block: read by the other workgroup of the block too -> no nontemporal hint
      p[ch] = __builtin_bit_cast(u32x4v, __builtin_amdgcn_raw_buffer_load_b128(rs, lane_bytes, ch * 256, HP == 2 ? 0 : 2));
  };
  // received bits of the two output tiles: 512 words each, wavefronts 0..7 look at the first, 8..15 at the second
  const u64 words_entry = ((wave < 8 ? e_lo : e_hi) >> 5) + (u64)((wave & 7) * 64);
  auto request_words = [&](int i) {
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc((void*)(a.masks + (u64)i * mrow + words_entry), 0, 256, 0x00020000);
    mw = __builtin_amdgcn_raw_buffer_load_b32(rs, lane * 4, 0, 0);
  };
  request(0, 0, NCH);
  request_words(0);

  // position of this lane's register r of array arr inside its output tile, in bytes of the mask and bit in the byte
  const int y_lane = ((lane >> 2) & 3) * 32 + (lane & 3) * 8 + ((lane >> 4) & 1) * 4 + (wave & 3) + (wave >> 2) * 128;
  // encoded values of both arrays -> wire rounding -> sum under the received bits
  auto finish = [&](float (&v)[R], int arr, const uint32_t* row, bool clean, float (&acc)[R]) {
    // one conversion per value with the result in the HIGH half (the low half converts a zero): that is the fp32
    // pattern of the rounded value, no unpacking
#pragma unroll
    for (int r = 0; r < R; ++r)
      v[r] = __builtin_bit_cast(float, pack_bf16x2(0.0f, scale_first ? v[r] * a.scale : v[r]));
    if (clean) {
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] += v[r];
    } else {
      unsigned off = (unsigned)sel * (unsigned)((e_hi - e_lo) >> 3) + ((y_lane + arr * 512) >> 3);
      asm volatile("" : "+v"(off));   // the address is formed here, on the rare path, not kept in registers all along
      const uint8_t* bytes = (const uint8_t*)row + (e_lo >> 3) + off;
      const uint32_t bit = 1u << (y_lane & 7);
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] += (bytes[r * 128] & bit) ? v[r] : 0.0f;
    }
  };

  bool all_clean = true;
  for (int i = 0; i < a.N; ++i) {
    const uint32_t* row = a.masks + (u64)i * mrow;
    const int nxt = i + 1 < a.N ? i + 1 : i;
    float X[R], Y[R];
    // The LDS addresses of the transforms depend on the lane alone; recomputing them each trip (a handful of
    // instructions) keeps them out of the registers that the trip needs for data
    int lane_t = lane;
    asm volatile("" : "+v"(lane_t));
    // The masks are rebuilt from the sign bytes for every worker (3 instructions a pair).  Left alone the compiler
    // computes all of them once before the loop -- and then has 32 registers too many and keeps them in scratch.
#pragma unroll
    for (int q = 0; q < NCH / 4; ++q) asm volatile("" : "+v"(sbytes[q]));
    // signs, then the first factor on the matrix cores
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const uint32_t byte = (sbytes[ch >> 2] >> (8 * (ch & 3))) & 0xFFu;
      u32x4v x = p[ch];
      x[0] ^= pair_sign_mask<0>(byte);
      x[1] ^= pair_sign_mask<1>(byte);
      x[2] ^= pair_sign_mask<2>(byte);
      x[3] ^= pair_sign_mask<3>(byte);
      const bf16x8v b = __builtin_bit_cast(bf16x8v, x);
      if constexpr (HP == 2) {
        const f32x4v d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hmat[0], b, f32x4v{0, 0, 0, 0}, 0, 0, 0);
        if (ch < 4) {
          X[4 * ch] = d[0]; X[4 * ch + 1] = d[1]; X[4 * ch + 2] = d[2]; X[4 * ch + 3] = d[3];
        } else {
          Y[4 * (ch & 3)] = d[0]; Y[4 * (ch & 3) + 1] = d[1]; Y[4 * (ch & 3) + 2] = d[2]; Y[4 * (ch & 3) + 3] = d[3];
        }
      } else {
        const f32x4v d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hmat[0], b, f32x4v{0, 0, 0, 0}, 0, 0, 0);
        const f32x4v d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hmat[HP == 2 ? 0 : 1], b, f32x4v{0, 0, 0, 0}, 0, 0, 0);
        X[4 * ch] = d0[0]; X[4 * ch + 1] = d0[1]; X[4 * ch + 2] = d0[2]; X[4 * ch + 3] = d0[3];
        Y[4 * ch] = d1[0]; Y[4 * ch + 1] = d1[1]; Y[4 * ch + 2] = d1[2]; Y[4 * ch + 3] = d1[3];
      }
    }
    const bool mine_clean = all_arrived(mw);   // a ballot: taken with every lane active, not inside the branch below
    if (lane == 0) s_clean[wave] = mine_clean ? 1u : 0u;   // read after the barrier inside the first transform
    // the next worker's loads travel during the transforms: half of them from here on, half after the first one
    request(nxt, 0, NCH / 2);
    request_words(nxt);
    if constexpr (HP == 2) {   // index bit 9: between the two arrays (2^15 blocks: done by the product)
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float s = X[r] + Y[r];
        Y[r] = X[r] - Y[r];
        X[r] = s;
      }
    }
    // left to do: register bits 2, 3 (index bits 7, 8), lane bits 0..3 (index bits 3..6), the wave bits (10..13)
    transform_dpp_sel<K, 0xC>(X, tbuf[flip], wave, lane_t);
    flip ^= 1;
    const bool clean = ((uint32_t)__builtin_amdgcn_ballot_w64(s_clean[lane_t & 15] != 0) & 0xFFFFu) == 0xFFFFu;
    all_clean = all_clean && clean;
    finish(X, 0, row, clean, accX);
    request(nxt, NCH / 2, NCH);
    transform_dpp_sel<K, 0xC>(Y, tbuf[flip], wave, lane_t);   // its barrier also orders s_clean
    flip ^= 1;
    finish(Y, 1, row, clean, accY);
  }
  __builtin_amdgcn_sched_barrier(0);

  // Received counts.  No worker lost anything in the two tiles (the common case): N everywhere.  Otherwise the mask
  // bytes of every worker are read once more here; the main loop carries no counters.
  uint32_t cntX[R / 4], cntY[R / 4];
#pragma unroll
  for (int r = 0; r < R / 4; ++r) cntX[r] = cntY[r] = 0;
  if (!all_clean) {
    for (int i = 0; i < a.N; ++i) {
      const unsigned off = (unsigned)sel * (unsigned)((e_hi - e_lo) >> 3) + (y_lane >> 3);
      const uint8_t* bytes = (const uint8_t*)(a.masks + (u64)i * mrow) + (e_lo >> 3) + off;
      const uint32_t bit = 1u << (y_lane & 7);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        cntX[r >> 2] += (bytes[r * 128] & bit) ? (1u << (8 * (r & 3))) : 0u;
        cntY[r >> 2] += (bytes[r * 128 + 64] & bit) ? (1u << (8 * (r & 3))) : 0u;
      }
    }
  }
  const int full = all_clean ? a.N : 0;
  if (a.total_out) {
    add_arrivals<R>(a.total_out, cntX, full);
    add_arrivals<R>(a.total_out, cntY, full);
  }
  // counts: gathered in LDS in entry order (the transform buffers are free now; both tiles, 32 KB), then two
  // 16-byte stores a lane
  auto store_counts_both = [&]() {
    if (!a.count_out) return;
    uint8_t* stage = (uint8_t*)&tbuf[0][0];
    __syncthreads();
    uint8_t* mine = stage + sel * T + y_lane;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      mine[r * 1024] = (uint8_t)count_of<R>(cntX, full, r);
      mine[r * 1024 + 512] = (uint8_t)count_of<R>(cntY, full, r);
    }
    __syncthreads();
    const u32x4v c_lo = ((const u32x4v*)stage)[threadIdx.x], c_hi = ((const u32x4v*)(stage + T))[threadIdx.x];
    __builtin_nontemporal_store(c_lo, (u32x4v*)(a.count_out + e_lo) + threadIdx.x);
    __builtin_nontemporal_store(c_hi, (u32x4v*)(a.count_out + e_hi) + threadIdx.x);
    __syncthreads();   // the staging area is part of the transform buffers: all reads before anyone transforms again
  };
  const float post = lane_sigma(lane, 4) * (scale_first ? 1.0f : a.scale);   // the sign that the DPP stages leave on a lane
  finalize_mean(accX, cntX, full, post);
  finalize_mean(accY, cntY, full, post);
  __syncthreads();   // every wavefront has read the last exchange of the loop before the buffers are used again

  // ---- decode: the plain transform of the mean over every index bit held here (bit 9 between the arrays, the
  // rest by position: lane bit 5 is the factor across the workgroup's two tiles)
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const float s = accX[r] + accY[r];
    accY[r] = accX[r] - accY[r];
    accX[r] = s;
  }
  if constexpr (HP == 1) store_counts_both();   // (never after the decoded tiles are stored: its barriers would wait for them)
  transform_transposed<K>(accX, tbuf[flip], tbuf[flip ^ 1], wave, lane);
  flip ^= 1;
  transform_transposed<K>(accY, tbuf[flip], tbuf[flip ^ 1], wave, lane);
  flip ^= 1;
  const float c = a.scale * sigma;
  // register r of array arr: decoded entry x_lane + arr*512 + (r>>2)*128 + (r&3) of a tile; the four registers of a
  // group are four consecutive entries: one 8-byte store, their signs one nibble of the sign stream
  const int x_lane = wave * 1024 + ((lane >> 2) & 3) * 32 + (lane & 3) * 8 + ((lane >> 4) & 1) * 4;
  auto store_decoded = [&](const float (&v)[R], int arr, u64 tile) {
    bf16_t* out = (bf16_t*)a.out + tile * T;
    const uint8_t* sb = sign_bytes + ((tile * T) >> 3);
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const int x = x_lane + arr * 512 + gq * 128;
      const uint32_t nib = ((uint32_t)sb[x >> 3] >> (x & 4)) & 0xFu;
      typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
      u32x2v o;
      o[0] = pack_bf16x2(v[4 * gq] * c, v[4 * gq + 1] * c) ^ pair_sign_mask<0>(nib);
      o[1] = pack_bf16x2(v[4 * gq + 2] * c, v[4 * gq + 3] * c) ^ pair_sign_mask<1>(nib);
      __builtin_nontemporal_store(o, (u32x2v*)(out + x));
    }
  };
  if constexpr (HP == 1) {
    store_decoded(accX, 0, t0 + sel);
    store_decoded(accY, 1, t0 + sel);
  } else {
    // This workgroup holds c_h, the decode over every index bit but 14; the block's tiles are
    //   index bit 14 = 0: c_0 + c_1   (tiles 0, 2)      index bit 14 = 1: c_0 - c_1   (tiles 1, 3)
    // Whoever of the two finishes first leaves c_h in its slot and is done; the other one takes it.  The hand-over
    // goes through memory with accesses that are coherent by themselves (system-scope atomics on 8-byte words:
    // written through, read past the caches), so that no cache-wide write-back or invalidation is needed.
    PairFlags* fl = (PairFlags*)a.count_in + blk;                     // count_in: the flags of this launch
    typedef unsigned long long w8;
    w8* slot_mine = (w8*)a.mean_out + (blk * 2 + h) * (u64)(2 * 8 * 1024);
    const w8* slot_other = (const w8*)a.mean_out + (blk * 2 + (h ^ 1)) * (u64)(2 * 8 * 1024);
    auto two = [](float x, float y) {
      return (w8)__builtin_bit_cast(uint32_t, x) | ((w8)__builtin_bit_cast(uint32_t, y) << 32);
    };
    if (threadIdx.x == 0) s_order = atomicAdd(&fl->arrived, 1u);
    __syncthreads();
    if (s_order == 0) {
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        __hip_atomic_store(slot_mine + g * 1024 + threadIdx.x, two(accX[2 * g], accX[2 * g + 1]), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
        __hip_atomic_store(slot_mine + (8 + g) * 1024 + threadIdx.x, two(accY[2 * g], accY[2 * g + 1]), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // waits for this wavefront's stores
      __syncthreads();
      if (threadIdx.x == 0) __hip_atomic_store(&fl->ready, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      store_counts_both();
      return;
    }
    // The other workgroup has passed its atomic, so it is running and will set `ready` whatever this one does:
    // the wait below ends.  It is bounded all the same, so that a wavefront can never spin for good.
    if (threadIdx.x == 0) {
      unsigned n = 0;
      while (__hip_atomic_load(&fl->ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) == 0 && ++n < kPairSpinLimit)
        __builtin_amdgcn_s_sleep(8);
    }
    __syncthreads();
    store_counts_both();
    const float sgn = h == 0 ? 1.0f : -1.0f;
    auto finish_pair = [&](float (&mine)[R], int arr) {
      float other[R];
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        const w8 t = __hip_atomic_load(slot_other + (arr * 8 + g) * 1024 + threadIdx.x, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_SYSTEM);
        other[2 * g] = __builtin_bit_cast(float, (uint32_t)t);
        other[2 * g + 1] = __builtin_bit_cast(float, (uint32_t)(t >> 32));
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float s = mine[r] + other[r];
        other[r] = sgn * (mine[r] - other[r]);
        mine[r] = s;
      }
      store_decoded(mine, arr, t0 + 2 * sel);
      store_decoded(other, arr, t0 + 2 * sel + 1);
    };
    finish_pair(accX, 0);
    finish_pair(accY, 1);
  }
}

}  // namespace ordev
