// OptiReduce gradient-bucket path: CPU ORACLE.  TEST INFRASTRUCTURE ONLY.
//
// This file is the slow, single-threaded, obviously-correct statement of what
// the GPU library computes.  It is linked by nothing in the product; only the
// tests, the smoke check and the benchmark's cpu_baseline leg may call it.
// It shares no code, header, table or constant generator with the HIP path.
//
// What it follows (OptiReduce, arXiv 2310.06993):
//   * Sec. 3.3 "Dispersing Gradient Loss": a *randomized* Hadamard transform is
//     applied to the gradient bucket before it is sharded and sent, and undone
//     after aggregation, so that a lost entry perturbs every decoded entry a
//     little instead of deleting one entry.
//   * Sec. 3.1.1 "TAR Algorithm": node r receives the r-th shard of every
//     worker and averages them; entries that the bounded transport did not
//     deliver are simply absent from that average (Sec. 1, third bullet: the
//     receiver still obtains an unbiased estimate; Sec. 3 overview).
//   * Sec. 4 "Implementation": encode runs on a bucket before reduction,
//     decode on the reduced bucket afterwards.
//
// Readings taken where the paper is silent (all listed in the design notes):
//   R1 random diagonal = Rademacher signs from Philox4x32-10 (Salmon et al.,
//      SC'11), keyed by a 64-bit seed that every worker shares; entry i of the
//      padded vector uses bit (i mod 128) of the 128-bit output for counter
//      (i div 128); bit set => multiply by -1.
//   R2 Hadamard matrix in Sylvester (natural) order, H[u][v]=(-1)^popcount(u&v).
//   R3 orthonormal scaling B^(-1/2) on encode and on decode.
//   R4 the transform is blockwise with block B = 2^k; a short last block is
//      zero padded before it is transformed; decode drops the pad.
//   R5 "average" = divide the sum of what arrived by how many arrived
//      (0 if nothing arrived).
//   R6 the slot of an entry that never arrived holds garbage and is never read.
//   R7 bf16 exists only at the memory/wire boundary (round to nearest even);
//      all interior arithmetic is wider.
//
// Arithmetic: every interior value is a double.  Values are rounded only where
// the three-call path has a memory boundary: the encoded shard (wire type), the
// per-entry sum (fp32), the mean handed to decode (fp32) and the decoded
// gradient (output type).  Sums over workers run in increasing worker order.
//
// Pins (tests/, CPU only): published Philox known-answer vectors; brute-force
// dense Hadamard products for every B <= 256 and against scipy's Sylvester
// construction; H(Hx) = Bx bit-exactly on integer data; Parseval; exact
// round trip with no drops; a hand-computed masked sum; the closed form for
// one lost encoded entry; linearity and the slice property of the sign stream;
// both decodes with a bf16 result against the dense product rounded once.
// Unpinned: the two MSE values the paper prints for its toy figure (the
// figure's vectors are not in the text)  ->  "parity unpinned" for that figure.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

// ---------------------------------------------------------------- Philox4x32-10
// Counter-based generator of Salmon, Moraes, Dror, Shaw (SC'11).  One call maps
// a 128-bit counter and a 64-bit key to 128 output bits through ten rounds.
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint32_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u;
  const uint32_t WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t pa = (uint64_t)MUL_A * c0;
    uint64_t pb = (uint64_t)MUL_B * c2;
    uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)pb;
    uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)pa;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += WEYL_A; k1 += WEYL_B;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Sign of padded-vector entry i under `seed` (reading R1): +1.0 or -1.0.
double rademacher(uint64_t seed, uint64_t i) {
  uint64_t q = i >> 7;
  uint32_t ctr[4] = {(uint32_t)q, (uint32_t)(q >> 32), 0u, 0u};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t w[4];
  philox4x32_10(ctr, key, w);
  unsigned bit = (unsigned)(i & 127u);
  return ((w[bit >> 5] >> (bit & 31u)) & 1u) ? -1.0 : 1.0;
}

// ------------------------------------------------------------------ bf16 <-> fp32
float bf16_to_float(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

// Round a float to bf16, nearest, ties to even; NaN stays NaN.
uint16_t float_to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
  uint32_t keep_lsb = (u >> 16) & 1u;
  u += 0x7FFFu + keep_lsb;
  return (uint16_t)(u >> 16);
}

// ------------------------------------------------- unnormalised Walsh-Hadamard
// In place, natural order: after the call x <- H x with H[u][v]=(-1)^popcount(u&v).
void hadamard_in_place(double* x, uint64_t len) {
  for (uint64_t stride = 1; stride < len; stride <<= 1)
    for (uint64_t base = 0; base < len; base += 2 * stride)
      for (uint64_t j = base; j < base + stride; ++j) {
        double a = x[j], b = x[j + stride];
        x[j] = a + b;
        x[j + stride] = a - b;
      }
}

uint64_t padded(uint64_t n, int k) {
  uint64_t B = (uint64_t)1 << k;
  return (n + B - 1) / B * B;
}

// Encode one vector (Sec. 3.3; readings R1-R4): y = B^(-1/2) H D x per block.
// load(i) returns entry i of the input as a double; store(i, v) receives the
// encoded entry i as a double and does the rounding to the wire type.
template <class Load, class Store>
void encode_generic(uint64_t n, int k, uint64_t seed, uint64_t base_index, Load load, Store store) {
  const uint64_t B = (uint64_t)1 << k;
  const uint64_t n_pad = padded(n, k);
  const double scale = 1.0 / std::sqrt((double)B);
  std::vector<double> blk(B);
  for (uint64_t start = 0; start < n_pad; start += B) {
    for (uint64_t j = 0; j < B; ++j) {
      uint64_t i = start + j;
      blk[j] = (i < n) ? rademacher(seed, base_index + i) * load(i) : 0.0;
    }
    hadamard_in_place(blk.data(), B);
    for (uint64_t j = 0; j < B; ++j) store(start + j, blk[j] * scale);
  }
}

// Decode (Sec. 3.3, Sec. 4; readings R1-R4): g = D B^(-1/2) H m per block,
// first n entries kept.
template <class Load, class Store>
void decode_generic(uint64_t n, int k, uint64_t seed, uint64_t base_index, Load load, Store store) {
  const uint64_t B = (uint64_t)1 << k;
  const uint64_t n_pad = padded(n, k);
  const double scale = 1.0 / std::sqrt((double)B);
  std::vector<double> blk(B);
  for (uint64_t start = 0; start < n_pad; start += B) {
    for (uint64_t j = 0; j < B; ++j) blk[j] = load(start + j);
    hadamard_in_place(blk.data(), B);
    for (uint64_t j = 0; j < B; ++j) {
      uint64_t i = start + j;
      if (i < n) store(i, rademacher(seed, base_index + i) * (blk[j] * scale));
    }
  }
}

bool mask_bit(const uint32_t* mask_row, uint64_t entry) {
  return (mask_row[entry >> 5] >> (entry & 31u)) & 1u;
}

// Masked aggregation at the node that owns a shard (Sec. 3.1.1; readings R5, R6):
// per entry, the sum over the workers whose copy arrived, and how many arrived.
template <class Load>
void masked_reduce_generic(const uint32_t* masks, int N, uint64_t L, Load load, float* sum_out,
                           uint8_t* count_out) {
  const uint64_t words = L / 32;
  for (uint64_t e = 0; e < L; ++e) {
    double acc = 0.0;
    unsigned cnt = 0;
    for (int i = 0; i < N; ++i)
      if (mask_bit(masks + (uint64_t)i * words, e)) {
        acc += load(i, e);
        ++cnt;
      }
    sum_out[e] = (float)acc;
    count_out[e] = (uint8_t)cnt;
  }
}

}  // namespace

extern "C" {

void orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  philox4x32_10(ctr, key, out);
}

// out[j] = 1 if padded-vector entry (first + j) is multiplied by -1, else 0.
void orc_sign_bits(uint64_t seed, uint64_t first, uint64_t count, uint8_t* out) {
  for (uint64_t j = 0; j < count; ++j) out[j] = rademacher(seed, first + j) < 0.0 ? 1 : 0;
}

uint64_t orc_padded_len(uint64_t n, int k) { return padded(n, k); }

void orc_hadamard_f64(double* x, uint64_t len) { hadamard_in_place(x, len); }

uint16_t orc_float_to_bf16(float f) { return float_to_bf16(f); }
float orc_bf16_to_float(uint16_t h) { return bf16_to_float(h); }

// ---- encode: fp32 in -> fp32 out; bf16 in -> bf16 out; and a double-precision
//      form with no rounding at all, used by the mathematical pins.
void orc_rht_encode_f64(const double* x, uint64_t n, int k, uint64_t seed, uint64_t base_index, double* out) {
  encode_generic(n, k, seed, base_index, [&](uint64_t i) { return x[i]; },
                 [&](uint64_t i, double v) { out[i] = v; });
}
void orc_rht_encode_f32(const float* x, uint64_t n, int k, uint64_t seed, uint64_t base_index, float* out) {
  encode_generic(n, k, seed, base_index, [&](uint64_t i) { return (double)x[i]; },
                 [&](uint64_t i, double v) { out[i] = (float)v; });
}
void orc_rht_encode_bf16(const uint16_t* x, uint64_t n, int k, uint64_t seed, uint64_t base_index, uint16_t* out) {
  encode_generic(n, k, seed, base_index, [&](uint64_t i) { return (double)bf16_to_float(x[i]); },
                 [&](uint64_t i, double v) { out[i] = float_to_bf16((float)v); });
}

// ---- masked aggregation
void orc_masked_reduce_f32(const float* shards, const uint32_t* masks, int N, uint64_t L, float* sum_out,
                           uint8_t* count_out) {
  masked_reduce_generic(masks, N, L, [&](int i, uint64_t e) { return (double)shards[(uint64_t)i * L + e]; },
                        sum_out, count_out);
}
void orc_masked_reduce_bf16(const uint16_t* shards, const uint32_t* masks, int N, uint64_t L, float* sum_out,
                            uint8_t* count_out) {
  masked_reduce_generic(masks, N, L,
                        [&](int i, uint64_t e) { return (double)bf16_to_float(shards[(uint64_t)i * L + e]); },
                        sum_out, count_out);
}

// ---- finalize (reading R5): mean of what arrived, 0 where nothing arrived.
void orc_finalize(const float* sum, const uint8_t* count, uint64_t L, float* mean_out) {
  for (uint64_t e = 0; e < L; ++e)
    mean_out[e] = count[e] ? (float)((double)sum[e] / (double)count[e]) : 0.0f;
}

// ---- decode: fp32 mean in -> fp32 / bf16 gradient out; and the unrounded form.
void orc_rht_decode_f64(const double* agg, uint64_t n, int k, uint64_t seed, uint64_t base_index, double* out) {
  decode_generic(n, k, seed, base_index, [&](uint64_t i) { return agg[i]; },
                 [&](uint64_t i, double v) { out[i] = v; });
}
void orc_rht_decode_f32(const float* agg, uint64_t n, int k, uint64_t seed, uint64_t base_index, float* out) {
  decode_generic(n, k, seed, base_index, [&](uint64_t i) { return (double)agg[i]; },
                 [&](uint64_t i, double v) { out[i] = (float)v; });
}
void orc_rht_decode_bf16(const float* agg, uint64_t n, int k, uint64_t seed, uint64_t base_index, uint16_t* out) {
  decode_generic(n, k, seed, base_index, [&](uint64_t i) { return (double)agg[i]; },
                 [&](uint64_t i, double v) { out[i] = float_to_bf16((float)v); });
}

// ---- second-stage loss (Sec. 3.1.1: the owner broadcasts its aggregated shard; Sec. 3.3: what is
//      lost there is spread over the block by the decode).  An aggregated entry whose bit is clear
//      never arrived and counts as zero; then decode as above.  mask: or_padded_len(n)/32 words.
void orc_rht_decode_masked_f32(const float* agg, const uint32_t* mask, uint64_t n, int k, uint64_t seed,
                               uint64_t base_index, float* out) {
  decode_generic(n, k, seed, base_index, [&](uint64_t i) { return mask_bit(mask, i) ? (double)agg[i] : 0.0; },
                 [&](uint64_t i, double v) { out[i] = (float)v; });
}
void orc_rht_decode_masked_bf16(const float* agg, const uint32_t* mask, uint64_t n, int k, uint64_t seed,
                                uint64_t base_index, uint16_t* out) {
  decode_generic(n, k, seed, base_index, [&](uint64_t i) { return mask_bit(mask, i) ? (double)agg[i] : 0.0; },
                 [&](uint64_t i, double v) { out[i] = float_to_bf16((float)v); });
}

// ---- loss monitoring (Sec. 3.4): how many (worker, entry) pairs arrived in this AllReduce;
//      the loss fraction is 1 - total / (N * L).
uint64_t orc_received_total(const uint8_t* count, uint64_t L) {
  uint64_t t = 0;
  for (uint64_t e = 0; e < L; ++e) t += count[e];
  return t;
}

// ---- second level of the hierarchical 2D scheme (Sec. 3.1.2, Appendix A): each group has already
//      aggregated its members into (sum, count); the partial aggregates of the groups that arrived
//      are combined, sums with sums and counts with counts.
void orc_masked_reduce_pairs(const float* sums, const uint8_t* counts, const uint32_t* masks, int G, uint64_t L,
                             float* sum_out, uint8_t* count_out) {
  const uint64_t words = L / 32;
  for (uint64_t e = 0; e < L; ++e) {
    double acc = 0.0;
    unsigned cnt = 0;
    for (int g = 0; g < G; ++g)
      if (mask_bit(masks + (uint64_t)g * words, e)) {
        acc += (double)sums[(uint64_t)g * L + e];
        cnt += counts[(uint64_t)g * L + e];
      }
    sum_out[e] = (float)acc;
    count_out[e] = (uint8_t)cnt;
  }
}

// ---- the whole path for one shard held by one node, as the composition of the
//      steps above with every memory-boundary rounding kept:
//      raw slices of N workers -> encode each -> masked sum/count -> mean -> decode.
//      L must be a multiple of 2^k.  count_out may be null.
void orc_fused_path_f32(const float* grads, const uint32_t* masks, int N, uint64_t L, int k, uint64_t seed,
                        uint64_t base_index, float* out, uint8_t* count_out) {
  std::vector<float> enc((uint64_t)N * L), sum(L), mean(L);
  std::vector<uint8_t> cnt(L);
  for (int i = 0; i < N; ++i)
    orc_rht_encode_f32(grads + (uint64_t)i * L, L, k, seed, base_index, enc.data() + (uint64_t)i * L);
  orc_masked_reduce_f32(enc.data(), masks, N, L, sum.data(), cnt.data());
  orc_finalize(sum.data(), cnt.data(), L, mean.data());
  orc_rht_decode_f32(mean.data(), L, k, seed, base_index, out);
  if (count_out) std::memcpy(count_out, cnt.data(), L);
}
void orc_fused_path_bf16(const uint16_t* grads, const uint32_t* masks, int N, uint64_t L, int k, uint64_t seed,
                         uint64_t base_index, uint16_t* out, uint8_t* count_out) {
  std::vector<uint16_t> enc((uint64_t)N * L);
  std::vector<float> sum(L), mean(L);
  std::vector<uint8_t> cnt(L);
  for (int i = 0; i < N; ++i)
    orc_rht_encode_bf16(grads + (uint64_t)i * L, L, k, seed, base_index, enc.data() + (uint64_t)i * L);
  orc_masked_reduce_bf16(enc.data(), masks, N, L, sum.data(), cnt.data());
  orc_finalize(sum.data(), cnt.data(), L, mean.data());
  orc_rht_decode_bf16(mean.data(), L, k, seed, base_index, out);
  if (count_out) std::memcpy(count_out, cnt.data(), L);
}

}  // extern "C"
