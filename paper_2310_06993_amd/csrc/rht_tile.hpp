// Device-side building blocks for the blockwise randomized Hadamard transform
// (OptiReduce, Sec. 3.3 "Dispersing Gradient Loss") on gfx950.
//
// Work is cut into TILES of 2^TL consecutive entries (TL = max(10, min(k, 14))).
// A tile is owned by one workgroup of W wavefronts; every lane holds R = 2^RL entries
// in registers (R = 16 or 32, W = 2^TL / (64 R)).  In both register layouts used here
// a register of a wavefront covers 64 CONSECUTIVE entries (lane l <-> entry l of that
// run), so
//   * every global load/store instruction of a wavefront is one 256-byte run,
//   * the 64 sign bits / 64 received bits of a register are two consecutive
//     32-bit words and can be used directly as a lane mask (no per-lane bit extraction).
//
// Layout A ("load" layout):  entry = wave*64R + reg*64 + lane
// Layout B ("wire" layout):  entry = (reg >> RLO)*64R + ((wave << RLO) + (reg & (2^RLO-1)))*64 + lane
// with RLO = RL - log2(W).  A and B differ by one exchange through LDS that swaps
// the wave bits with the top register bits; for W = 1 they are the same layout.
//
// Butterfly stages (the Hadamard factors commute, so any order is the same map):
//   entry bits 0..5   : across lanes (DPP, ds_swizzle, ds_bpermute)
//   register bits     : plain add/sub between registers
//   wave bits         : become register bits after the LDS exchange
//
// Lane stages for entry bits 0, 1, 3 (DPP) and 4, 5 (LDS crossbar) use
// v <- v + s*neighbour with s = +1 on the lower lane of a pair and -1 on the upper one
// (one v_fmac_f32, with a DPP source where a DPP pattern exists), which leaves the
// *negated* difference on the upper lane.  All later stages combine values that sit on
// the same lane, so the result of a whole transform is H x multiplied, on lane l, by
// parity(l & SIGMA_BITS).  That per-lane factor ("sigma") is folded into the scale
// multiply that follows.  The stage for bit 2 (no single DPP pattern gives lane^4 on
// gfx9) is a masked add / subtract pair with row_shl:4 / row_shr:4 and is exact in sign.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ordev {

typedef unsigned long long u64;

// Entries per lane: 16, except 32 in the "wide" form of 2^13 and 2^14 blocks (a 64 KB tile then needs 8
// wavefronts, so two workgroups fit on a CU).  Measured on MI355X against each other: for 2^14 the encode,
// decode and fused kernels came out 3-5 % faster with 16 entries per lane (16 wavefronts), the reduce+decode
// kernel 5 % faster with 32.
constexpr int kWide = 1000;   // Geo<K + kWide>: the same block size with 32 entries per lane

// Geometry for a block of 2^K entries.  KT bits are transformed inside a tile; for
// K > 14 the remaining HB bits are handled by combining 2^HB input tiles with +-1
// before the in-tile transform (H_{2^K} = H_{2^HB} (x) H_{2^14}).
// K == 0 stands for "any block_log2 <= 10, taken at run time" (one wavefront per tile).
template <int KSEL>
struct Geo {
  static constexpr int K = KSEL % kWide;
  static constexpr bool WIDE = KSEL >= kWide;
  static_assert(!WIDE || K == 13 || K == 14, "the wide form exists for blocks of 2^13 and 2^14 entries only");
  static constexpr int KT = (K == 0) ? 10 : (K > 14 ? 14 : K);
  static constexpr int TL = KT;
  static constexpr int T = 1 << TL;
  static constexpr int RL = WIDE ? 5 : 4;
  static constexpr int R = 1 << RL;
  static constexpr int Q = TL - 6 - RL;          // wave bits
  static_assert(Q >= 0 && Q <= 4 && Q <= RL, "unsupported tile geometry");
  static constexpr int W = 1 << Q;
  static constexpr int THREADS = 64 * W;
  static constexpr int HB = (K > 14) ? K - 14 : 0;
  static constexpr int PARTS = 1 << HB;
  static constexpr int RLO = RL - Q;
  static constexpr int WAVE_ENTRIES = 64 * R;
};

__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

template <int K>
__device__ __forceinline__ int off_a(int wave, int reg) { return wave * Geo<K>::WAVE_ENTRIES + reg * 64; }
template <int K>
__device__ __forceinline__ int off_b(int wave, int reg) {
  constexpr int RLO = Geo<K>::RLO;
  return (reg >> RLO) * Geo<K>::WAVE_ENTRIES + (((wave << RLO) + (reg & ((1 << RLO) - 1))) * 64);
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
template <> __device__ __forceinline__ uint8_t from_f32<uint8_t>(float v) { return (uint8_t)(int)v; }
template <bool NT> __device__ __forceinline__ void store_one(float* p, float v) {
  if (NT) __builtin_nontemporal_store(v, p); else *p = v;
}
template <bool NT> __device__ __forceinline__ void store_one(uint8_t* p, uint8_t v) {
  if (NT) __builtin_nontemporal_store(v, p); else *p = v;
}
template <bool NT> __device__ __forceinline__ void store_one(bf16_t* p, bf16_t v) {
  if (NT) __builtin_nontemporal_store(v.bits, &p->bits); else p->bits = v.bits;
}
template <bool NT> __device__ __forceinline__ float load_one(const float* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT> __device__ __forceinline__ uint8_t load_one(const uint8_t* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT> __device__ __forceinline__ bf16_t load_one(const bf16_t* p) {
  return bf16_t{NT ? __builtin_nontemporal_load(&p->bits) : p->bits};
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

// Sign lane-masks for the NR registers of this wavefront in layout A.  `g` is the index, in the
// padded vector, of the wavefront's first entry (a multiple of 128).  Entry i flips sign iff bit
// (i mod 128) of Philox(counter = i div 128, key = seed) is set.  Lanes 0..NR/2-1 each produce the
// 128 bits of one counter; the words move to scalar registers with readlane.
template <int NR>
__device__ __forceinline__ void sign_masks(u64 seed, u64 g, u64 (&sg)[NR]) {
  u64 ctr = (g >> 7) + (u64)lane_id();
  u32x4 w = philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)((r & 1) ? w.c : w.a), r >> 1);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)((r & 1) ? w.d : w.b), r >> 1);
    sg[r] = (u64)lo | ((u64)hi << 32);
  }
}

__device__ __forceinline__ bool in_mask(u64 m) { return __builtin_amdgcn_inverse_ballot_w64(m); }

template <int NR>
__device__ __forceinline__ void apply_signs(float (&v)[NR], const u64 (&sg)[NR]) {
#pragma unroll
  for (int r = 0; r < NR; ++r) v[r] = in_mask(sg[r]) ? -v[r] : v[r];
}

// ------------------------------------------------------------------ butterflies
#define OR_IO16(v, o)                                                                                          \
  "+v"(v[o + 0]), "+v"(v[o + 1]), "+v"(v[o + 2]), "+v"(v[o + 3]), "+v"(v[o + 4]), "+v"(v[o + 5]),                \
      "+v"(v[o + 6]), "+v"(v[o + 7]), "+v"(v[o + 8]), "+v"(v[o + 9]), "+v"(v[o + 10]), "+v"(v[o + 11]),          \
      "+v"(v[o + 12]), "+v"(v[o + 13]), "+v"(v[o + 14]), "+v"(v[o + 15])
#define OR_FMAC_DPP(i, ctrl) "v_fmac_f32_dpp %" #i ", %" #i ", %16 " ctrl " row_mask:0xf bank_mask:0xf\n\t"
// v[o+r] += s * (v[o+r] of the partner lane selected by the DPP control), r = 0..15.  The leading s_nop
// covers the two wait states a DPP read needs after a VALU write of the same register; inside the block
// every instruction touches a different register.
#define OR_FMAC_DPP16(v, o, s, ctrl)                                                                         \
  asm("s_nop 1\n\t" OR_FMAC_DPP(0, ctrl) OR_FMAC_DPP(1, ctrl) OR_FMAC_DPP(2, ctrl) OR_FMAC_DPP(3, ctrl)        \
          OR_FMAC_DPP(4, ctrl) OR_FMAC_DPP(5, ctrl) OR_FMAC_DPP(6, ctrl) OR_FMAC_DPP(7, ctrl)                  \
              OR_FMAC_DPP(8, ctrl) OR_FMAC_DPP(9, ctrl) OR_FMAC_DPP(10, ctrl) OR_FMAC_DPP(11, ctrl)            \
                  OR_FMAC_DPP(12, ctrl) OR_FMAC_DPP(13, ctrl) OR_FMAC_DPP(14, ctrl) OR_FMAC_DPP(15, ctrl)      \
      : OR_IO16(v, o)                                                                                        \
      : "v"(s))

// lane ^ 4 butterfly, exact: lanes with bit 2 clear get v[l] + v[l+4], the others v[l-4] - v[l]
#define OR_X4(o, i)                                                                  \
  "v_add_f32_dpp %" #o ", %" #i ", %" #i " row_shl:4 row_mask:0xf bank_mask:0x5\n\t" \
  "v_sub_f32_dpp %" #o ", %" #i ", %" #i " row_shr:4 row_mask:0xf bank_mask:0xa\n\t"
__device__ __forceinline__ void lane_xor4_exact8(float* v) {
  float t0, t1, t2, t3, t4, t5, t6, t7;
  asm("s_nop 1\n\t" OR_X4(0, 8) OR_X4(1, 9) OR_X4(2, 10) OR_X4(3, 11) OR_X4(4, 12) OR_X4(5, 13) OR_X4(6, 14) OR_X4(7, 15)
      : "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3), "=&v"(t4), "=&v"(t5), "=&v"(t6), "=&v"(t7)
      : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]));
  v[0] = t0; v[1] = t1; v[2] = t2; v[3] = t3; v[4] = t4; v[5] = t5; v[6] = t6; v[7] = t7;
}

// lane bits whose stage leaves the negated difference on the upper lane
constexpr int SIGMA_BITS = 0x3B;

template <int BIT, int NR>
__device__ __forceinline__ void lane_stage(float (&v)[NR], int lane) {
  const float s = (lane >> BIT) & 1 ? -1.0f : 1.0f;
  if constexpr (BIT == 0) {
    OR_FMAC_DPP16(v, 0, s, "quad_perm:[1,0,3,2]");
    if constexpr (NR == 32) OR_FMAC_DPP16(v, 16, s, "quad_perm:[1,0,3,2]");
  } else if constexpr (BIT == 1) {
    OR_FMAC_DPP16(v, 0, s, "quad_perm:[2,3,0,1]");
    if constexpr (NR == 32) OR_FMAC_DPP16(v, 16, s, "quad_perm:[2,3,0,1]");
  } else if constexpr (BIT == 2) {
#pragma unroll
    for (int o = 0; o < NR; o += 8) lane_xor4_exact8(&v[o]);
  } else if constexpr (BIT == 3) {
    OR_FMAC_DPP16(v, 0, s, "row_ror:8");
    if constexpr (NR == 32) OR_FMAC_DPP16(v, 16, s, "row_ror:8");
  } else {
    const int a32 = (lane ^ 32) << 2;
    // in chunks of 8 registers, so that at most 8 partner values are live at a time
#pragma unroll
    for (int o = 0; o < NR; o += 8) {
#pragma unroll
      for (int r = o; r < o + 8; ++r) {
        int i = __builtin_bit_cast(int, v[r]);
        int p = BIT == 4 ? __builtin_amdgcn_ds_swizzle(i, 0x401F) : __builtin_amdgcn_ds_bpermute(a32, i);
        v[r] = __builtin_fmaf(__builtin_bit_cast(float, p), s, v[r]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// all lane stages for entry bits 0..nbits-1 (nbits uniform, <= 6)
template <int NR>
__device__ __forceinline__ void lane_stages(float (&v)[NR], int lane, int nbits) {
  static_assert(NR == 16 || NR == 32, "16 or 32 entries per lane");
  if (nbits > 0) lane_stage<0>(v, lane);
  if (nbits > 1) lane_stage<1>(v, lane);
  if (nbits > 2) lane_stage<2>(v, lane);
  if (nbits > 3) lane_stage<3>(v, lane);
  if (nbits > 4) lane_stage<4>(v, lane);
  if (nbits > 5) lane_stage<5>(v, lane);
}

// +1 / -1 factor left on this lane by `nbits` lane stages
__device__ __forceinline__ float lane_sigma(int lane, int nbits) {
  return (__builtin_popcount(lane & ((1 << nbits) - 1) & SIGMA_BITS) & 1) ? -1.0f : 1.0f;
}

template <int RBIT, int NR>
__device__ __forceinline__ void reg_stage(float (&v)[NR]) {
  constexpr int S = 1 << RBIT;
  if constexpr (S < NR) {
#pragma unroll
    for (int r = 0; r < NR; ++r)
      if ((r & S) == 0) {
        float a = v[r], b = v[r + S];
        v[r] = a + b;
        v[r + S] = a - b;
      }
  }
}

// register stages for register-index bits lo..hi-1 (uniform run-time range inside 0..5)
template <int NR>
__device__ __forceinline__ void reg_stages(float (&v)[NR], int lo, int hi) {
  if (lo <= 0 && hi > 0) reg_stage<0>(v);
  if (lo <= 1 && hi > 1) reg_stage<1>(v);
  if (lo <= 2 && hi > 2) reg_stage<2>(v);
  if (lo <= 3 && hi > 3) reg_stage<3>(v);
  if (lo <= 4 && hi > 4) reg_stage<4>(v);
}

// LDS exchange between the two layouts (W > 1 only).  xbuf holds one tile of floats, indexed in
// layout-B order: slot = (wave_b*R + reg_b)*64 + lane.  PRE_SYNC = false is for callers that alternate
// between two buffers: a buffer is then rewritten only after every wavefront has passed the barrier of
// the exchange in between, i.e. after all its readers are done.
template <int K, bool A_TO_B, bool PRE_SYNC>
__device__ __forceinline__ void exchange(float (&v)[Geo<K>::R], float* xbuf, int wave, int lane) {
  constexpr int Q = Geo<K>::Q, RLO = Geo<K>::RLO, R = Geo<K>::R;
  static_assert(Q > 0, "exchange needs more than one wavefront");
  if (PRE_SYNC) __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    // layout A register r of wave `wave` is layout B register ((wave << RLO) | r_lo) of wave (r >> RLO)
    int slot_cross = (((r >> RLO) * R) + ((wave << RLO) | (r & ((1 << RLO) - 1)))) * 64 + lane;
    int slot_own = (wave * R + r) * 64 + lane;
    if (A_TO_B) xbuf[slot_cross] = v[r]; else xbuf[slot_own] = v[r];
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    int slot_cross = (((r >> RLO) * R) + ((wave << RLO) | (r & ((1 << RLO) - 1)))) * 64 + lane;
    int slot_own = (wave * R + r) * 64 + lane;
    v[r] = A_TO_B ? xbuf[slot_own] : xbuf[slot_cross];
  }
}

// Unscaled Hadamard transform of one tile over its low `kt` entry bits.  A_TO_B: layout A in, layout B
// out; else layout B in, layout A out (the same linear map either way).  The result on lane l carries
// the factor lane_sigma(l, min(kt, 6)).
template <int K, bool A_TO_B, bool PRE_SYNC = true>
__device__ __forceinline__ void transform(float (&v)[Geo<K>::R], float* xbuf, int wave, int lane, int kt) {
  constexpr int Q = Geo<K>::Q, RL = Geo<K>::RL;
  lane_stages(v, lane, kt < 6 ? kt : 6);
  reg_stages(v, 0, kt <= 6 ? 0 : (kt < 6 + RL ? kt - 6 : RL));
  if constexpr (Q > 0) {
    exchange<K, A_TO_B, PRE_SYNC>(v, xbuf, wave, lane);
    reg_stages(v, RL - Q, RL);
  }
}

// ------------------------------------------------------------------ transform with transposed lane bits
// For tiles of W = 2, 4, 8 or 16 wavefronts x 16 registers (2^11 ... 2^14 entries).
// On MI355X a plain add/sub issues at twice the rate of anything with a DPP control, so the stages of lane
// bits 2..5 cost three times a register stage (and those of bits 4, 5 an LDS-crossbar operation each on
// top).  Here those four bits are made register bits by a transposition inside the wavefront (through a
// part of LDS that belongs to the wavefront alone: no barrier) and run as register stages; only lane
// bits 0, 1 use DPP.  Result on lane l times tr_sigma(l).
//   1. register stages (entry bits 6..9), DPP stages (bits 0, 1)
//   2. transposition: register r, lane l  ->  register (l >> 2), lane (l & 3) | (r << 2);
//      rows of 68 floats make the write (bank 4r + l) and the read (bank 4(l' >> 2) + (l' & 3) + 4r') hit
//      64 different banks
//   3. register stages (entry bits 2..5)
//      now wavefront w, register r', lane l' holds entry (l' & 3) | r' << 2 | rho << 6 | w << 10 of the tile,
//      rho = l' >> 2 the register the value sat in before step 2
//   4. exchange between wavefronts, written straight to layout-B positions (Q = log2 W, RLO = 4 - Q):
//      wavefront rho >> RLO, register (rho & (2^RLO - 1)) | w << RLO, lane (l' & 3) | r' << 2.
//      Register rows are 68 floats apart (64 when RLO = 0) and the parts of the wavefronts 16 * 68 + 4 * 2^RLO,
//      so that the 64 lanes of a store fall into 64 different banks; so do those of a load
//   5. register stages RLO..3 (entry bits 10 and up)
// Layout A in, layout B out -- or layout B in, layout A out: with 16 registers a lane the two exchanges are
// the same map of (wavefront, register, lane); only the entry bits that the positions stand for differ, and
// every index bit is transformed exactly once either way.
// `ta` and `tb` are two buffers of tr_floats<K> floats; the caller swaps them from one call to the next, which
// leaves one barrier per call: the transposition is written into the wavefront's own part of `ta` (last
// read by this wavefront, in the exchange of the call before), the exchange into `tb` (last read as the
// transposition buffer of the call before, by its owner, ahead of that call's barrier).
constexpr int TR_ROW = 68;   // floats per register row
template <int K> constexpr int tr_wave = 16 * TR_ROW + (4 << Geo<K>::RLO);   // part of a wavefront
template <int K> constexpr int tr_floats = Geo<K>::W * tr_wave<K>;
__device__ __forceinline__ float tr_sigma(int lane) { return (__builtin_popcount(lane & 3) & 1) ? -1.0f : 1.0f; }

template <int K>
__device__ __forceinline__ void transform_transposed(float (&v)[16], float* ta, float* tb, int wave, int lane) {
  // rows of the exchange: 68 floats apart where register bits come from the lane index (banks), else 64,
  // which lets two rows share one LDS instruction (the st64 forms)
  constexpr int RLO = Geo<K>::RLO, PART = tr_wave<K>, XROW = RLO ? TR_ROW : 64;
  static_assert(Geo<K>::R == 16 && Geo<K>::Q >= 1 && Geo<K>::Q <= 4, "2, 4, 8 or 16 wavefronts of 16 registers");
  reg_stages(v, 0, 4);
  lane_stage<0>(v, lane);
  lane_stage<1>(v, lane);
  float* mine = ta + wave * PART;
#pragma unroll
  for (int r = 0; r < 16; ++r) mine[r * TR_ROW + lane] = v[r];
  __builtin_amdgcn_wave_barrier();
  const float* back = mine + (lane >> 2) * TR_ROW + (lane & 3);
#pragma unroll
  for (int r = 0; r < 16; ++r) v[r] = back[r * 4];
  reg_stages(v, 0, 4);
  const int rho = lane >> 2;
  float* to = tb + (rho >> RLO) * PART + ((rho & ((1 << RLO) - 1)) + (wave << RLO)) * XROW + (lane & 3);
#pragma unroll
  for (int r = 0; r < 16; ++r) to[r * 4] = v[r];
  __syncthreads();
  const float* from = tb + wave * PART + lane;
#pragma unroll
  for (int r = 0; r < 16; ++r) v[r] = from[r * XROW];
  reg_stages(v, RLO, 4);
}

// ------------------------------------------------------------------ tile loads / stores
// `p` points at entry 0 of the vector, `e0` is the tile's first entry, `limit` the number of valid
// entries of the vector; entries at or beyond `limit` read as zero / are not written.  FULL = true
// promises e0 + tile <= limit.
// A tile that may be cut short by `limit` goes through raw buffer accesses: the descriptor covers exactly
// the valid bytes of the tile, so the hardware range check returns 0 for loads beyond it and drops stores
// beyond it -- no per-lane compares or exec masks.
template <class T>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const T* p, u64 e0, u64 limit) {
  const u64 left = limit > e0 ? (limit - e0) * sizeof(T) : 0;
  const int bytes = left > 0x7FFFFFFFull ? 0x7FFFFFFF : (int)left;
  return __builtin_amdgcn_make_buffer_rsrc((void*)(p + e0), 0, bytes, 0x00020000);
}
__device__ __forceinline__ float buf_load(__amdgpu_buffer_rsrc_t r, int entry, const float*) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, entry * 4, 0, 0));
}
__device__ __forceinline__ float buf_load(__amdgpu_buffer_rsrc_t r, int entry, const bf16_t*) {
  return __builtin_bit_cast(float, (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, entry * 2, 0, 0) << 16);
}
__device__ __forceinline__ float buf_load(__amdgpu_buffer_rsrc_t r, int entry, const uint8_t*) {
  return (float)__builtin_amdgcn_raw_buffer_load_b8(r, entry, 0, 0);
}
__device__ __forceinline__ void buf_store(__amdgpu_buffer_rsrc_t r, int entry, float v, float*) {
  __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, entry * 4, 0, 0);
}
__device__ __forceinline__ void buf_store(__amdgpu_buffer_rsrc_t r, int entry, float v, bf16_t*) {
  __builtin_amdgcn_raw_buffer_store_b16(from_f32<bf16_t>(v).bits, r, entry * 2, 0, 0);
}
__device__ __forceinline__ void buf_store(__amdgpu_buffer_rsrc_t r, int entry, float v, uint8_t*) {
  __builtin_amdgcn_raw_buffer_store_b8(from_f32<uint8_t>(v), r, entry, 0, 0);
}

// NT = true: nontemporal loads, for inputs that are read once.  Measured on MI355X: 4-7 % faster for the
// N-to-1 shard kernels.
template <int K, bool LAYOUT_B, bool FULL, bool NT = false, class T>
__device__ __forceinline__ void load_tile(const T* __restrict__ p, u64 e0, u64 limit, int wave, int lane,
                                          float (&v)[Geo<K>::R]) {
  constexpr int R = Geo<K>::R;
  if (FULL || e0 + Geo<K>::T <= limit) {
    // uniform base (scalar registers) + 32-bit lane offset
    const T* q = p + e0;
    const unsigned l = (unsigned)lane;
#pragma unroll
    for (int r = 0; r < R; ++r)
      v[r] = to_f32(load_one<NT>(&(q + (LAYOUT_B ? off_b<K>(wave, r) : off_a<K>(wave, r)))[l]));
  } else {
    const __amdgpu_buffer_rsrc_t rs = tile_rsrc(p, e0, limit);
#pragma unroll
    for (int r = 0; r < R; ++r)
      v[r] = buf_load(rs, (LAYOUT_B ? off_b<K>(wave, r) : off_a<K>(wave, r)) + lane, (const T*)nullptr);
  }
}

// NT = true: nontemporal stores.  Measured on MI355X: faster when reads dominate the kernel's traffic
// (the N-to-1 shard kernels), slower for the 1:1 encode / decode kernels.
template <int K, bool LAYOUT_B, bool FULL, bool NT = false, class T>
__device__ __forceinline__ void store_tile(T* __restrict__ p, u64 e0, u64 limit, int wave, int lane,
                                           const float (&v)[Geo<K>::R]) {
  constexpr int R = Geo<K>::R;
  if (FULL || e0 + Geo<K>::T <= limit) {
    T* q = p + e0;
    const unsigned l = (unsigned)lane;
#pragma unroll
    for (int r = 0; r < R; ++r)
      store_one<NT>(&(q + (LAYOUT_B ? off_b<K>(wave, r) : off_a<K>(wave, r)))[l], from_f32<T>(v[r]));
  } else {
    const __amdgpu_buffer_rsrc_t rs = tile_rsrc(p, e0, limit);
#pragma unroll
    for (int r = 0; r < R; ++r)
      buf_store(rs, (LAYOUT_B ? off_b<K>(wave, r) : off_a<K>(wave, r)) + lane, v[r], (T*)nullptr);
  }
}

// Received bits of one worker for this wavefront's R registers in layout B, as ONE vector register:
// lane l < 2R holds the 32-bit word for entries 32*(l&1) .. +31 of register l>>1 (lanes at or above 2R
// repeat lanes 0..2R-1).  `row` = that worker's mask row (bit j of word w = entry 32w+j), `e0` = tile's
// first entry, `limit` = shard length (multiple of 32).  Words wholly beyond `limit` read as 0.  A
// vector load (rather than a scalar one) so that it is in flight together with the tile data and costs
// no scalar registers.
template <int K>
__device__ __forceinline__ int mask_word_offset(int wave, int lane) {
  const int l = lane & (2 * Geo<K>::R - 1);
  return (off_b<K>(wave, l >> 1) >> 5) + (l & 1);
}
template <int K, bool FULL>
__device__ __forceinline__ uint32_t load_mask_words(const uint32_t* __restrict__ row, u64 e0, u64 limit, int word_off) {
  if (FULL) return (row + (e0 >> 5))[(unsigned)word_off];
  const u64 w = (e0 >> 5) + (u64)word_off;
  return (w << 5) < limit ? row[w] : 0u;
}
// true iff every entry of the wavefront's tile part arrived
__device__ __forceinline__ bool all_arrived(uint32_t words) {
  return __builtin_amdgcn_ballot_w64(words != 0xFFFFFFFFu) == 0;
}
// the 64 received bits of register r as a lane mask
__device__ __forceinline__ u64 mask_of_reg(uint32_t words, int r) {
  uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)words, 2 * r);
  uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)words, 2 * r + 1);
  return (u64)lo | ((u64)hi << 32);
}

}  // namespace ordev
