// The fused path (OptiReduce Sec. 3.3 encode, Sec. 3.1.1 aggregation, Sec. 3.3 / Sec. 4 decode) for bf16
// gradients in blocks of 2^15 / 2^16 entries: PARTS = 2 / 4 tiles of 2^14 entries per block.
//
// As in k_fused_pairs a workgroup of 16 wavefronts produces TWO output tiles of its block, p_lo = h and
// p_hi = h + PARTS/2, from one reading of the block's input tiles (H_{2P} = [[H_P, H_P], [H_P, -H_P]]).
// What differs:
//   * Memory is touched 16 bytes a lane.  A wavefront's 1024 entries of a tile are two runs of 512; register
//     c*8 + j of lane l holds entry c*512 + l*8 + j ("layout S"), so a lane's 8 registers of a run are one
//     16-byte load of bf16, and a decoded run is one 16-byte store.  The butterflies do not care which index
//     bit sits where as long as every bit is transformed once; what changes is what a position means:
//         before the transform  (wave w, register r, lane l)  is entry  w*1024 + (r>>3)*512 + l*8 + (r&7)
//         after it              (wave w, register r, lane l)  is entry  r*1024 + (w>>3)*512 + l*8 + (w&7)
//     (the transform swaps the index bits held by the register number with those held by the wave number).
//   * The sign lane masks still come from a table read with scalar loads; k_sign_table_strided writes it in
//     layout-S order (word r of a wavefront's slice: bit l = sign of entry (r>>3)*512 + l*8 + (r&7)).
//   * After the transform a register covers 64 entries 8 apart, so the received bits of a register are bit
//     (w&7) of 64 consecutive bytes of the mask.  The common case is decided for the whole workgroup at once
//     (every bit of both output tiles set: plain adds); otherwise each lane fetches its byte per register.
//   * Four tiles per block: the two workgroups of a block no longer hand the mean to a second launch.  The
//     one that finishes first leaves its two partial decodes' inputs (a = m_h + m_{h+2}, b = m_h - m_{h+2}) in
//     the workspace and exits; the other one combines them with its own and decodes all four tiles.
#pragma once
#include "rht_kernels.hpp"

namespace ordev {

typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));

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
  unsigned ready;     // set by the first one once its partial sums are in the workspace
};
constexpr unsigned kPairSpinLimit = 1u << 22;   // polls of `ready` before the waiting workgroup gives up

template <int K>
__global__ __launch_bounds__(1024) void k_fused_wide(PathArgs a) {
  constexpr int T = Geo<K>::T, R = 16, HB = Geo<K>::HB, PARTS = Geo<K>::PARTS, HP = PARTS / 2;
  static_assert(Geo<K>::R == 16 && Geo<K>::W == 16 && (PARTS == 2 || PARTS == 4), "2^14 tiles, two or four per block");
  __shared__ float tbuf[2][tr_floats<K>];
  __shared__ uint32_t s_clean[16];
  __shared__ unsigned s_order;
  int flip = 0;
  const int wave = wave_id(), lane = lane_id();
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
  const u64 e_lo = (t0 + h) * T, e_hi = (t0 + h + HP) * T;
  const bf16_t* grads = (const bf16_t*)a.in;
  const float sigma = tr_sigma(lane);
  constexpr bool scale_first = (K & 1);   // 2^(-k/2) is a power of two for even k and commutes with the rounding
  const u64 mrow = L >> 5;
  typedef const u64 __attribute__((address_space(4))) * table_ptr;

  float acc_lo[R], acc_hi[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc_lo[r] = acc_hi[r] = 0.0f;

  // one input tile's slice of this wavefront: two 16-byte loads a lane
  auto request = [&](int i, int q, u32x4v (&p)[2]) {
    const u32x4v* src = (const u32x4v*)(grads + (u64)i * L + (t0 + q) * T + (u64)wave * 1024);
    // Four tiles per block: the other workgroup of the block reads the same tiles a little earlier or later and
    // should find them in the L2 (measured: 1.17 x the algorithmic bytes fetched against 1.56 x with the
    // nontemporal hint, and 7 % less time).  Two tiles per block: read once, nontemporal.
    if constexpr (HP == 2) {
      p[0] = src[lane];
      p[1] = src[64 + lane];
    } else {
      p[0] = __builtin_nontemporal_load(src + lane);
      p[1] = __builtin_nontemporal_load(src + 64 + lane);
    }
  };
  // dst (+)= +-(signed tile q).  The sign words of a tile are loaded here, where the tile is used, and the
  // results are pinned here, so that the words of only one group of tiles are live at a time.
  auto add_signed = [&](float (&dst)[R], const u32x4v (&p)[2], int q, bool negate, bool first) {
    table_ptr sg = (table_ptr)(a.sign_tab + ((((t0 + q) * T) + (u64)wave * 1024) >> 6));
    if constexpr (HP == 2) asm volatile("" : "+s"(sg));
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const uint32_t w = p[r >> 3][(r & 7) >> 1];
      const float t = (r & 1) ? bf16_hi(w) : bf16_lo(w);
      const bool flipped = in_mask(sg[r]);
      const float ts = negate ? (flipped ? t : -t) : (flipped ? -t : t);
      dst[r] = first ? ts : dst[r] + ts;
    }
  };
#define OR_PIN16(v) asm volatile("" : OR_IO16(v, 0))
  // encoded values of one output tile -> wire rounding -> sum under the received bits.
  // `tile_e` = first entry of the output tile in the shard, `row` = this worker's mask row.
  auto finish_tile = [&](float (&v)[R], u64 tile_e, const uint32_t* row, bool clean, float (&acc)[R]) {
#pragma unroll
    for (int r = 0; r < R; r += 2) {
      const uint32_t pk = scale_first ? pack_bf16x2(v[r] * a.scale, v[r + 1] * a.scale) : pack_bf16x2(v[r], v[r + 1]);
      v[r] = bf16_lo(pk);
      v[r + 1] = bf16_hi(pk);
    }
    if (clean) {
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] += v[r];
    } else {
      // register r of this wavefront: entries r*1024 + (wave>>3)*512 + lane*8 + (wave&7), i.e. bit (wave&7) of
      // byte r*128 + (wave>>3)*64 + lane of the tile's part of the row
      const uint8_t* bytes = (const uint8_t*)row + (tile_e >> 3) + (wave >> 3) * 64 + lane;
      const uint32_t bit = 1u << (wave & 7);
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] += (bytes[r * 128] & bit) ? v[r] : 0.0f;
    }
  };

  // The next worker's tiles (packed, half the registers of their unpacked form) travel while this worker's two
  // transforms run: the tiles of A are asked for before the first transform, those of C after it, when A's
  // registers are free.  The requests inside the loop are unconditional -- the last trip asks for the last
  // worker again -- so that the number of loads in flight is the same on every path into a wait.
  u32x4v p0[2], p1[2], p2[2], p3[2];
  uint32_t mw;
  // received bits of the two output tiles: 512 words each, wavefronts 0..7 look at p_lo, 8..15 at p_hi
  const uint32_t* my_words = a.masks + ((wave < 8 ? e_lo : e_hi) >> 5) + (u64)((wave & 7) * 64 + lane);
  request(0, 0, p0);
  if constexpr (HP == 2) request(0, 1, p1);
  mw = my_words[0];
  request(0, HP, p2);
  if constexpr (HP == 2) request(0, HP + 1, p3);
  bool all_clean_lo = true, all_clean_hi = true;
  for (int i = 0; i < a.N; ++i) {
    const uint32_t* row = a.masks + (u64)i * mrow;
    const int nxt = i + 1 < a.N ? i + 1 : i;
    float A[R], C[R];
    add_signed(A, p0, 0, false, true);
    if constexpr (HP == 2) add_signed(A, p1, 1, part_coef(h, 1) < 0.0f, false);
    OR_PIN16(A);
    const bool mine_clean = all_arrived(mw);   // a ballot: taken with every lane active, not inside the branch below
    if (lane == 0) s_clean[wave] = mine_clean ? 1u : 0u;   // read after the barrier inside the first transform
    request(nxt, 0, p0);
    if constexpr (HP == 2) request(nxt, 1, p1);
    mw = my_words[(u64)nxt * mrow];
    add_signed(C, p2, HP, false, true);
    if constexpr (HP == 2) add_signed(C, p3, HP + 1, part_coef(h, 1) < 0.0f, false);
    OR_PIN16(C);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float s = A[r] + C[r];
      C[r] = A[r] - C[r];
      A[r] = s;
    }
    transform_transposed<K>(A, tbuf[flip], tbuf[flip ^ 1], wave, lane);
    flip ^= 1;
    const uint32_t flags = (uint32_t)__builtin_amdgcn_ballot_w64(s_clean[lane & 15] != 0);
    const bool clean_lo = (flags & 0xFFu) == 0xFFu, clean_hi = (flags & 0xFF00u) == 0xFF00u;
    all_clean_lo = all_clean_lo && clean_lo;
    all_clean_hi = all_clean_hi && clean_hi;
    finish_tile(A, e_lo, row, clean_lo, acc_lo);
    request(nxt, HP, p2);
    if constexpr (HP == 2) request(nxt, HP + 1, p3);
    transform_transposed<K>(C, tbuf[flip], tbuf[flip ^ 1], wave, lane);   // its barrier also orders s_clean for the next worker
    flip ^= 1;
    finish_tile(C, e_hi, row, clean_hi, acc_hi);
  }
  __builtin_amdgcn_sched_barrier(0);

  // Received counts.  No worker lost anything in the tile (the common case): N everywhere.  Otherwise the mask
  // bytes of every worker are read once more here; the main loop carries no counters.
  uint32_t cnt_lo[R / 4], cnt_hi[R / 4];
  auto recount = [&](u64 tile_e, bool all_clean, uint32_t (&cnt)[R / 4]) {
#pragma unroll
    for (int r = 0; r < R / 4; ++r) cnt[r] = 0;
    if (all_clean) return;
    const uint32_t bit = 1u << (wave & 7);
    for (int i = 0; i < a.N; ++i) {
      const uint8_t* bytes = (const uint8_t*)(a.masks + (u64)i * mrow) + (tile_e >> 3) + (wave >> 3) * 64 + lane;
#pragma unroll
      for (int r = 0; r < R; ++r) cnt[r >> 2] += (bytes[r * 128] & bit) ? (1u << (8 * (r & 3))) : 0u;
    }
  };
  recount(e_lo, all_clean_lo, cnt_lo);
  recount(e_hi, all_clean_hi, cnt_hi);
  const int full_lo = all_clean_lo ? a.N : 0, full_hi = all_clean_hi ? a.N : 0;
  if (a.total_out) {
    add_arrivals<R>(a.total_out, cnt_lo, full_lo);
    add_arrivals<R>(a.total_out, cnt_hi, full_hi);
  }
  // counts: gathered in LDS in entry order (the transform buffers are free now), then one 16-byte store a lane
  auto store_tile_counts = [&](u64 tile_e, const uint32_t (&cnt)[R / 4], int full) {
    if (!a.count_out) return;
    uint8_t* stage = (uint8_t*)&tbuf[0][0];
    __syncthreads();
    uint8_t* mine = stage + (wave >> 3) * 512 + lane * 8 + (wave & 7);
#pragma unroll
    for (int r = 0; r < R; ++r) mine[r * 1024] = (uint8_t)count_of<R>(cnt, full, r);
    __syncthreads();
    const u32x4v c16 = ((const u32x4v*)stage)[threadIdx.x];
    __builtin_nontemporal_store(c16, (u32x4v*)(a.count_out + tile_e) + threadIdx.x);
  };
  const float post = sigma * (scale_first ? 1.0f : a.scale);
  finalize_mean(acc_lo, cnt_lo, full_lo, post);
  finalize_mean(acc_hi, cnt_hi, full_hi, post);
  // the factor across the pair of tiles
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const float s = acc_lo[r] + acc_hi[r];
    acc_hi[r] = acc_lo[r] - acc_hi[r];
    acc_lo[r] = s;
  }
  const float c = a.scale * sigma;
  // v = mean-domain tile in the after-transform positions -> decoded tile q of the block, stored 16 bytes a lane
  auto decode_tile = [&](float (&v)[R], int q) {
    transform_transposed<K>(v, tbuf[flip], tbuf[flip ^ 1], wave, lane);
    flip ^= 1;
    table_ptr sg = (table_ptr)(a.sign_tab + ((((t0 + q) * T) + (u64)wave * 1024) >> 6));
    u32x4v o[2];
#pragma unroll
    for (int r = 0; r < R; r += 2) {
      const float x0 = v[r] * c, x1 = v[r + 1] * c;
      o[r >> 3][(r & 7) >> 1] = pack_bf16x2(in_mask(sg[r]) ? -x0 : x0, in_mask(sg[r + 1]) ? -x1 : x1);
    }
    u32x4v* dst = (u32x4v*)((bf16_t*)a.out + (t0 + q) * T + (u64)wave * 1024);
    __builtin_nontemporal_store(o[0], dst + lane);
    __builtin_nontemporal_store(o[1], dst + 64 + lane);
  };
  // (Where the counts are stored: their staging needs barriers, and a barrier waits for the wavefront's
  // outstanding stores.  So never after the decoded tiles have been stored -- the workgroup would sit there until
  // memory has taken them -- and not before the hand-over either, whose own wait they would lengthen.)
  if constexpr (HP == 1) {
    store_tile_counts(e_lo, cnt_lo, full_lo);
    store_tile_counts(e_hi, cnt_hi, full_hi);
    decode_tile(acc_lo, 0);
    decode_tile(acc_hi, 1);
  } else {
    // a = acc_lo, b = acc_hi of this workgroup (h); the block's tiles are
    //   0: a_0 + a_1   1: a_0 - a_1   2: b_0 + b_1   3: b_0 - b_1
    // Whoever of the two finishes first leaves (a, b) in its slot and is done; the other one takes them.
    // The hand-over goes through memory with accesses that are coherent by themselves (written through and read
    // past the caches: system-scope atomics on 8-byte words), so that no cache-wide write-back or invalidation is
    // needed -- a device-wide fence here makes a wavefront flush and drop the whole L2 of its XCD, which every
    // other workgroup pays for.  Order: a wavefront's stores are complete at the barrier, the flag is set after it.
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
        __hip_atomic_store(slot_mine + g * 1024 + threadIdx.x, two(acc_lo[2 * g], acc_lo[2 * g + 1]), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
        __hip_atomic_store(slot_mine + (8 + g) * 1024 + threadIdx.x, two(acc_hi[2 * g], acc_hi[2 * g + 1]), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // waits for this wavefront's stores
      __syncthreads();
      if (threadIdx.x == 0) __hip_atomic_store(&fl->ready, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      store_tile_counts(e_lo, cnt_lo, full_lo);
      store_tile_counts(e_hi, cnt_hi, full_hi);
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
    const float sgn = h == 0 ? 1.0f : -1.0f;
    auto finish_pair = [&](float (&mine)[R], int which, int q_sum, int q_diff) {
      float other[R];
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        const w8 t = __hip_atomic_load(slot_other + (which * 8 + g) * 1024 + threadIdx.x, __ATOMIC_RELAXED,
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
      decode_tile(mine, q_sum);
      decode_tile(other, q_diff);
    };
    store_tile_counts(e_lo, cnt_lo, full_lo);
    store_tile_counts(e_hi, cnt_hi, full_hi);
    finish_pair(acc_lo, 0, 0, 1);
    finish_pair(acc_hi, 1, 2, 3);
  }
}

}  // namespace ordev
