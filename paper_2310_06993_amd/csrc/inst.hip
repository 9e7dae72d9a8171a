// One block-size class of kernels (compile with -DOR_K=0, 11, 12, ... 16).
#include "launch_table.hpp"
#if OR_K > 14
#include "rht_fused_mx.hpp"
#endif

#ifndef OR_K
#error "compile with -DOR_K=<class>"
#endif

namespace orhost {
using namespace ordev;

namespace {
constexpr int K = OR_K;
typedef Geo<K> G;

#define OR_LAUNCHER_T(name, kernel, threads)                                                 \
  /* serves output tiles a.unit0 .. a.unit0 + units - 1, one workgroup per tile */          \
  hipError_t name(const PathArgs& a, unsigned long long units, hipStream_t s, int pos) {    \
    if (units == 0) return hipSuccess;                                                       \
    if (units > 0x7FFFFFFFull) return hipErrorInvalidValue;                                  \
    return launch_kernel(kernel, dim3((unsigned)units), dim3(threads), s, pos, a);           \
  }
#define OR_LAUNCHER(name, kernel) OR_LAUNCHER_T(name, kernel, G::THREADS)

// blocks above 2^14: one workgroup per block of G::PARTS tiles; a.unit0 and units count tiles
#define OR_BLOCK_LAUNCHER(name, kernel)                                                      \
  hipError_t name(const PathArgs& a, unsigned long long units, hipStream_t s, int pos) {    \
    const unsigned long long blocks = units >> G::HB;                                        \
    if (blocks == 0) return hipSuccess;                                                      \
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;                                 \
    return launch_kernel(kernel, dim3((unsigned)blocks), dim3(G::THREADS), s, pos, a);       \
  }

#define OR_SPLIT_LAUNCHER(name, LAUNCHER, kernel_full, kernel_tail)                          \
  LAUNCHER(name##_full, kernel_full)                                                         \
  LAUNCHER(name##_tail, kernel_tail)                                                         \
  /* a.unit0 = number of leading tiles that need no bounds checks; the rest go to the checked kernel */ \
  hipError_t name(const PathArgs& a, unsigned long long units, hipStream_t s, int pos) {    \
    const unsigned long long nfull = a.unit0 < units ? a.unit0 : units, ntail = units - nfull; \
    PathArgs b = a;                                                                          \
    b.unit0 = 0;                                                                             \
    if (nfull) {                                                                             \
      if (hipError_t e = name##_full(b, nfull, s, ntail ? (pos & LAUNCH_FIRST) : pos)) return e; \
    }                                                                                        \
    if (ntail) {                                                                             \
      b.unit0 = nfull;                                                                       \
      return name##_tail(b, ntail, s, nfull ? (pos & LAUNCH_LAST) : pos);                    \
    }                                                                                        \
    return hipSuccess;                                                                       \
  }

#if OR_K <= 14
#define OR_ENC(In, Wire, FULL) (k_encode<K, In, Wire, FULL>)
#define OR_DEC(Out, FIN, FULL, MASKED) (k_decode<K, Out, FIN, FULL, MASKED>)
#define OR_XFORM_LAUNCHER OR_LAUNCHER
#else
#define OR_ENC(In, Wire, FULL) (k_encode_block<K, In, Wire, FULL>)
#define OR_DEC(Out, FIN, FULL, MASKED) (k_decode_block<K, Out, FIN, FULL, MASKED>)
#define OR_XFORM_LAUNCHER OR_BLOCK_LAUNCHER
#endif
OR_SPLIT_LAUNCHER(enc_f32, OR_XFORM_LAUNCHER, OR_ENC(float, float, true), OR_ENC(float, float, false))
OR_SPLIT_LAUNCHER(enc_bf16, OR_XFORM_LAUNCHER, OR_ENC(bf16_t, bf16_t, true), OR_ENC(bf16_t, bf16_t, false))
OR_SPLIT_LAUNCHER(dec_f32, OR_XFORM_LAUNCHER, OR_DEC(float, false, true, false), OR_DEC(float, false, false, false))
OR_SPLIT_LAUNCHER(dec_bf16, OR_XFORM_LAUNCHER, OR_DEC(bf16_t, false, true, false), OR_DEC(bf16_t, false, false, false))
OR_SPLIT_LAUNCHER(fdec_f32, OR_XFORM_LAUNCHER, OR_DEC(float, true, true, false), OR_DEC(float, true, false, false))
OR_SPLIT_LAUNCHER(fdec_bf16, OR_XFORM_LAUNCHER, OR_DEC(bf16_t, true, true, false), OR_DEC(bf16_t, true, false, false))
OR_SPLIT_LAUNCHER(mdec_f32, OR_XFORM_LAUNCHER, OR_DEC(float, false, true, true), OR_DEC(float, false, false, true))
OR_SPLIT_LAUNCHER(mdec_bf16, OR_XFORM_LAUNCHER, OR_DEC(bf16_t, false, true, true), OR_DEC(bf16_t, false, false, true))
#if OR_K <= 14
// reduce+decode of 2^13 and 2^14 blocks keeps 32 entries per lane
constexpr int KR = (K == 13 || K == 14) ? K + kWide : K;
OR_LAUNCHER_T(rdec_f32, (k_reduce_decode<KR, float, float>), Geo<KR>::THREADS)
OR_LAUNCHER_T(rdec_bf16, (k_reduce_decode<KR, bf16_t, bf16_t>), Geo<KR>::THREADS)
// several buckets per launch: `units` = tiles of all the buckets together
#define OR_BATCH_LAUNCHER(name, kernel, threads)                                             \
  hipError_t name(const BatchArgs& a, unsigned long long units, hipStream_t s, int pos) {   \
    if (units == 0) return hipSuccess;                                                       \
    if (units > 0x7FFFFFFFull) return hipErrorInvalidValue;                                  \
    return launch_kernel(kernel, dim3((unsigned)units), dim3(threads), s, pos, a);           \
  }
OR_BATCH_LAUNCHER(rdecb_f32, (k_reduce_decode_batched<KR, float>), Geo<KR>::THREADS)
OR_BATCH_LAUNCHER(rdecb_bf16, (k_reduce_decode_batched<KR, bf16_t>), Geo<KR>::THREADS)
OR_BATCH_LAUNCHER(fdecb_f32, (k_finalize_decode_batched<K, float>), G::THREADS)
OR_BATCH_LAUNCHER(fdecb_bf16, (k_finalize_decode_batched<K, bf16_t>), G::THREADS)
// The fused kernels come in two forms where a lane holds 16 entries: with a second tile buffer (the next
// worker's tile travels while this one is transformed), which shortens the chain of dependent steps of a
// workgroup and wins while a launch puts at most three workgroups on each of the 256 CUs, and without,
// which wins beyond that (measured on MI355X; same arithmetic, same results).
// (Tiles of 8 or 16 wavefronts, at most two workgroups on a CU whatever the grid: always the first form.)
constexpr unsigned long long kPrefetchUpTo = (G::W >= 8) ? ~0ull : 3 * 256;
constexpr bool kTwoForms = (G::R == 16);
#define OR_FUSED_LAUNCHER(name, Args, kernel)                                                \
  hipError_t name(const Args& a, unsigned long long units, hipStream_t s, int pos) {        \
    if (units == 0) return hipSuccess;                                                       \
    if (units > 0x7FFFFFFFull) return hipErrorInvalidValue;                                  \
    if (kTwoForms && units <= kPrefetchUpTo)                                                 \
      return launch_kernel(kernel<K, OR_FUSED_IN, kTwoForms>, dim3((unsigned)units), dim3(G::THREADS), s, pos, a); \
    return launch_kernel(kernel<K, OR_FUSED_IN, false>, dim3((unsigned)units), dim3(G::THREADS), s, pos, a); \
  }
#define OR_FUSED_IN float
OR_FUSED_LAUNCHER(fus_f32, PathArgs, k_fused)
OR_FUSED_LAUNCHER(fusb_f32, BatchArgs, k_fused_batched)
#undef OR_FUSED_IN
#define OR_FUSED_IN bf16_t
OR_FUSED_LAUNCHER(fus_bf16, PathArgs, k_fused)
OR_FUSED_LAUNCHER(fusb_bf16, BatchArgs, k_fused_batched)
#undef OR_FUSED_IN
#else
// one workgroup per pair of output tiles; `units` = output tiles of the shard
#define OR_PAIR_LAUNCHER(name, kernel)                                                       \
  hipError_t name(const PathArgs& a, unsigned long long units, hipStream_t s, int pos) {    \
    if (units == 0) return hipSuccess;                                                       \
    const unsigned long long blocks = units >> G::HB, per = G::PARTS / 2;                    \
    unsigned long long grid = per == 1 ? blocks : (blocks + 7) / 8 * 8 * per;                \
    if (grid > 0x7FFFFFFFull) return hipErrorInvalidValue;                                   \
    return launch_kernel(kernel, dim3((unsigned)grid), dim3(G::THREADS), s, pos, a);         \
  }
OR_PAIR_LAUNCHER(fus_f32, (k_fused_pairs<K, float>))
OR_PAIR_LAUNCHER(fus_bf16, (k_fused_mx<K>))
#endif
}  // namespace

#if !defined(__HIP_DEVICE_COMPILE__)
#define OR_CAT2(a, b) a##b
#define OR_CAT(a, b) OR_CAT2(a, b)
extern const KernelTable OR_CAT(or_kernel_table_, OR_K) = {
    G::TL, enc_f32, enc_bf16, dec_f32, dec_bf16, fdec_f32, fdec_bf16, mdec_f32, mdec_bf16,
#if OR_K <= 14
    rdec_f32, rdec_bf16,
#else
    nullptr, nullptr,
#endif
    fus_f32, fus_bf16,
#if OR_K <= 14
    fusb_f32, fusb_bf16, rdecb_f32, rdecb_bf16, fdecb_f32, fdecb_bf16
#else
    nullptr, nullptr, nullptr, nullptr, nullptr, nullptr
#endif
};
#endif

}  // namespace orhost
