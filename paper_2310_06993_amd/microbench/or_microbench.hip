// Measurements behind the design choices of liboptireduce_hip on MI355X (gfx950).  Not part of the library:
// a standalone program (python -m paper_2310_06993_amd.build --microbench builds it next to this file).
//
//     ./or_microbench [streams] [issue] [overlap] [front] [dot2] [reread]      (no argument: everything)
//
// Every kernel is in bounds and self-contained; each variant is a kernel of its own name, so that
// `rocprofv3 --kernel-trace --stats -- ./or_microbench` lists one average duration per variant.
//   streams  what HBM delivers to the traffic mixes of the path: read-only, 8 reads : 1 write (plain and
//            nontemporal stores), copy; at 100 MB and 1.3 GB
//   issue    issue cost of the vector instructions the kernels are made of (ns per wave64 instruction per SIMD,
//            four wavefronts per SIMD), and of the bf16 / fp32 matrix-core instructions
//   overlap  whether matrix-core work of some wavefronts of a SIMD runs under vector work of the others
//   front    the first Hadamard factor of the bf16 fused kernel for 2^16 blocks (64 raw bf16 entries a lane in,
//            32 fp32 a lane out: unpack, sign flip, +-1 combination of four tiles, three butterfly stages) in its
//            vector form and as a bf16 matrix-core product with the signs applied by XOR on packed pairs
//   dot2     v_dot2c_f32_bf16 as "unpack and add": cost, and whether it equals an fp32 addition bit for bit
//   reread   a workgroup reading 128 KB chunks R times in a row, with 16-byte and with 2-byte loads
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <vector>

typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d (%s) at line %d\n", (int)e_, hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

static float time_ms(void (*launch)(void*), void* ctx, int reps) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  launch(ctx);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  for (int i = 0; i < reps; ++i) launch(ctx);
  CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  CK(hipEventDestroy(e0)); CK(hipEventDestroy(e1));
  return ms / reps;
}

// ------------------------------------------------------------------ streams
// MODE 0 read only, 1 eight reads : one write, 2 the same with nontemporal stores, 3 copy.  MB names the size.
// One 16-byte access per lane and step; a workgroup walks 8 consecutive 4 KB pieces (the eight "workers" of the
// 8:1 mix are eight rows, as in the path).
template <int MODE, int MB>
__global__ __launch_bounds__(256) void mb_stream(const u4* __restrict__ src, u4* __restrict__ dst, size_t row16) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= row16) return;
  u4 acc = {0, 0, 0, 0};
  if (MODE == 3) {
#pragma unroll
    for (int r = 0; r < 8; ++r) dst[(size_t)r * row16 + i] = src[(size_t)r * row16 + i];
    return;
  }
  u4 v[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) v[r] = __builtin_nontemporal_load(src + (size_t)r * row16 + i);
#pragma unroll
  for (int r = 0; r < 8; ++r) acc ^= v[r];
  if (MODE == 1) dst[i] = acc;
  else if (MODE == 2) __builtin_nontemporal_store(acc, dst + i);
  else if (acc[0] == 0x12345678u && acc[1] == 0x9ABCDEF0u) dst[i] = acc;   // never true for the zero-filled input
}
// Consecutive launches of the 100 MB cases walk through the 1.4 GB buffers, so that none finds its data in the
// 256 MB last-level cache from the launch before.
template <int MODE, int MB> struct StreamCtx { const u4* s; u4* d; size_t row16; int turn; };
template <int MODE, int MB> static void launch_stream(void* c) {
  auto* x = (StreamCtx<MODE, MB>*)c;
  const size_t slices = (size_t)1400 * (1 << 20) / 16 / (8 * x->row16);
  const size_t off = (size_t)(x->turn++ % (int)slices) * 8 * x->row16;
  hipLaunchKernelGGL((mb_stream<MODE, MB>), dim3((unsigned)((x->row16 + 255) / 256)), dim3(256), 0, 0, x->s + off, x->d + off,
                     x->row16);
}
template <int MODE, int MB> static void run_stream(const u4* s, u4* d, const char* what) {
  const size_t row16 = (size_t)MB * 1000000 / 8 / 16;     // eight rows make MB megabytes of reads
  StreamCtx<MODE, MB> c = {s, d, row16, 0};
  const float ms = time_ms(launch_stream<MODE, MB>, &c, 20);
  const double rd = 8.0 * row16 * 16, wr = MODE == 0 ? 0 : (MODE == 3 ? rd : row16 * 16.0);
  printf("  %-34s %5d MB read: %8.1f us  %6.0f GB/s (read + written bytes)\n", what, MB, ms * 1e3, (rd + wr) / ms / 1e6);
}
static void streams() {
  printf("streams (HBM peak 8000 GB/s):\n");
  const size_t bytes = (size_t)1400 << 20;
  u4 *s, *d;
  CK(hipMalloc(&s, bytes)); CK(hipMalloc(&d, bytes));
  CK(hipMemset(s, 0, bytes)); CK(hipMemset(d, 0, bytes));
  run_stream<0, 100>(s, d, "read only");
  run_stream<0, 1300>(s, d, "read only");
  run_stream<1, 100>(s, d, "8 reads : 1 write");
  run_stream<1, 1300>(s, d, "8 reads : 1 write");
  run_stream<2, 100>(s, d, "8 reads : 1 write, nontemporal");
  run_stream<2, 1300>(s, d, "8 reads : 1 write, nontemporal");
  run_stream<3, 100>(s, d, "copy");
  run_stream<3, 1300>(s, d, "copy");
  CK(hipFree(s)); CK(hipFree(d));
}

// ------------------------------------------------------------------ issue costs
enum { OP_ADD, OP_FMA, OP_XOR, OP_ADD_DPP, OP_CNDMASK_SGPR, OP_LSHL, OP_CVT_PK_BF16, OP_MUL_LO, OP_DOT2C, OP_MFMA_BF16, OP_MFMA_F32,
       OP_DPP_ROR8, OP_DPP_SHL4, OP_DPP_MIRROR, OP_DPP_HALF_MIRROR, OP_SWIZZLE, OP_COUNT };
static const char* op_name[OP_COUNT] = {"v_add_f32", "v_fma_f32", "v_xor_b32", "v_add_f32 (DPP quad_perm)", "v_cndmask_b32 (SGPR mask, neg)",
                                        "v_lshlrev_b32", "v_cvt_pk_bf16_f32", "v_mul_lo_u32", "v_dot2c_f32_bf16",
                                        "v_mfma_f32_16x16x32_bf16", "v_mfma_f32_16x16x4_f32", "v_add_f32 (DPP row_ror:8)",
                                        "v_add_f32 (DPP row_shl:4, bank-masked)", "v_add_f32 (DPP row_mirror)",
                                        "v_add_f32 (DPP row_half_mirror)", "ds_swizzle_b32 (lane ^ 4) + v_add_f32"};
template <int OP>
__global__ __launch_bounds__(1024) void mb_issue(float* out, int iters, unsigned long long mask) {
  float v[16];
  f4 c[4];
  bf8 a, b;
  for (int j = 0; j < 8; ++j) { a[j] = (__bf16)1.0f; b[j] = (__bf16)(float)(threadIdx.x & 3); }
  for (int i = 0; i < 4; ++i) c[i] = f4{0, 0, 0, 0};
  for (int i = 0; i < 16; ++i) v[i] = threadIdx.x * 1e-3f + i;
  const float s = (threadIdx.x & 1) ? -1.0f : 1.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if (OP == OP_ADD) v[i] = v[i] + s;
        else if (OP == OP_FMA) v[i] = __builtin_fmaf(v[i], s, s);
        else if (OP == OP_XOR) asm volatile("v_xor_b32_e32 %0, %1, %0" : "+v"(v[i]) : "v"(s));
        else if (OP == OP_ADD_DPP) asm volatile("v_add_f32_dpp %0, %0, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "+v"(v[i]) : "v"(s));
        else if (OP == OP_CNDMASK_SGPR) asm volatile("v_cndmask_b32_e64 %0, %0, -%0, %1" : "+v"(v[i]) : "s"(mask));
        else if (OP == OP_LSHL) asm volatile("v_lshlrev_b32_e32 %0, 1, %0" : "+v"(v[i]));
        else if (OP == OP_CVT_PK_BF16) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(v[i]) : "v"(s));
        else if (OP == OP_MUL_LO) asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(v[i]) : "v"(s));
        else if (OP == OP_DOT2C) v[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, 0x3F803F80u), __builtin_bit_cast(bf2, 0x00003F80u), v[i], false);
        else if (OP == OP_DPP_ROR8) asm volatile("v_add_f32_dpp %0, %0, %1 row_ror:8 row_mask:0xf bank_mask:0xf" : "+v"(v[i]) : "v"(s));
        else if (OP == OP_DPP_SHL4) asm volatile("v_add_f32_dpp %0, %0, %1 row_shl:4 row_mask:0xf bank_mask:0x5" : "+v"(v[i]) : "v"(s));
        else if (OP == OP_DPP_MIRROR) asm volatile("v_add_f32_dpp %0, %0, %1 row_mirror row_mask:0xf bank_mask:0xf" : "+v"(v[i]) : "v"(s));
        else if (OP == OP_DPP_HALF_MIRROR) asm volatile("v_add_f32_dpp %0, %0, %1 row_half_mirror row_mask:0xf bank_mask:0xf" : "+v"(v[i]) : "v"(s));
        else if (OP == OP_SWIZZLE) v[i] = v[i] + __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v[i]), 0x101F));
        else if (OP == OP_MFMA_BF16) { if ((i & 7) == 0) c[(r * 2 + i / 8) & 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c[(r * 2 + i / 8) & 3], 0, 0, 0); }
        else if (OP == OP_MFMA_F32) { if ((i & 7) == 0) c[(r * 2 + i / 8) & 3] = __builtin_amdgcn_mfma_f32_16x16x4f32(s, v[0], c[(r * 2 + i / 8) & 3], 0, 0, 0); }
      }
    __builtin_amdgcn_sched_barrier(0);
  }
  float t = 0;
  for (int i = 0; i < 16; ++i) t += v[i];
  for (int i = 0; i < 4; ++i) t += c[i][0] + c[i][1] + c[i][2] + c[i][3];
  out[blockIdx.x * 1024 + threadIdx.x] = t;
}
struct IssueCtx { float* out; int iters; };
template <int OP> static void launch_issue(void* c) {
  auto* x = (IssueCtx*)c;
  hipLaunchKernelGGL((mb_issue<OP>), dim3(256), dim3(1024), 0, 0, x->out, x->iters, 0x5555AAAA3333CCCCull);
}
template <int OP> static void run_issue(float* out) {
  IssueCtx c = {out, 500};
  const float ms = time_ms(launch_issue<OP>, &c, 3);
  const int per_iter = (OP == OP_MFMA_BF16 || OP == OP_MFMA_F32) ? 32 : 256;
  const double ns = ms * 1e6 / c.iters / per_iter / 4;    // four wavefronts per SIMD share it
  printf("  %-34s %6.2f ns per instruction per SIMD (%5.1f clocks at 2.4 GHz)\n", op_name[OP], ns, ns * 2.4);
}
static void issue(float* out) {
  printf("issue cost, one workgroup of 16 wavefronts per CU (four per SIMD), long unrolled bodies:\n");
  run_issue<OP_ADD>(out); run_issue<OP_FMA>(out); run_issue<OP_XOR>(out); run_issue<OP_ADD_DPP>(out);
  run_issue<OP_CNDMASK_SGPR>(out); run_issue<OP_LSHL>(out); run_issue<OP_CVT_PK_BF16>(out); run_issue<OP_MUL_LO>(out);
  run_issue<OP_DOT2C>(out); run_issue<OP_MFMA_BF16>(out); run_issue<OP_MFMA_F32>(out);
  run_issue<OP_DPP_ROR8>(out); run_issue<OP_DPP_SHL4>(out); run_issue<OP_DPP_MIRROR>(out); run_issue<OP_DPP_HALF_MIRROR>(out);
  run_issue<OP_SWIZZLE>(out);
}

// ------------------------------------------------------------------ overlap of matrix-core and vector work
// MODE 0: every wavefront 256 v_add_f32 per trip.  1: every wavefront 32 bf16 products per trip.  2: wavefronts
// 0-3, 8-11 the vector work and 4-7, 12-15 the products (two of each kind on every SIMD), half the trips each kind
// would need alone.  F32: the fp32 product 16x16x4 instead.
template <int MODE, bool F32>
__global__ __launch_bounds__(1024) void mb_overlap(float* out, int iters) {
  bf8 a, b;
  for (int j = 0; j < 8; ++j) { a[j] = (__bf16)1.0f; b[j] = (__bf16)(float)(threadIdx.x & 3); }
  f4 c[4];
  float v[16];
  for (int i = 0; i < 4; ++i) c[i] = f4{0, 0, 0, 0};
  for (int i = 0; i < 16; ++i) v[i] = threadIdx.x * 1e-3f + i;
  const int wave = threadIdx.x >> 6;
  const bool do_m = MODE == 1 || (MODE == 2 && (wave & 4));
  const bool do_v = MODE == 0 || (MODE == 2 && !(wave & 4));
  for (int it = 0; it < iters; ++it) {
    if (do_m) {
#pragma unroll
      for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          c[i] = F32 ? __builtin_amdgcn_mfma_f32_16x16x4f32(v[0], v[1], c[i], 0, 0, 0)
                     : __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c[i], 0, 0, 0);
    }
    if (do_v) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = v[i] + (r & 1 ? 1.0f : -1.0f) * v[(i + 1) & 15];
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  float s = 0;
  for (int i = 0; i < 4; ++i) s += c[i][0] + c[i][1] + c[i][2] + c[i][3];
  for (int i = 0; i < 16; ++i) s += v[i];
  out[blockIdx.x * 1024 + threadIdx.x] = s;
}
template <int MODE, bool F32> static void launch_overlap(void* c) {
  auto* x = (IssueCtx*)c;
  hipLaunchKernelGGL((mb_overlap<MODE, F32>), dim3(256), dim3(1024), 0, 0, x->out, x->iters);
}
template <bool F32> static void run_overlap(float* out) {
  IssueCtx c = {out, 500};
  const float v = time_ms(launch_overlap<0, F32>, &c, 3), m = time_ms(launch_overlap<1, F32>, &c, 3),
              h = time_ms(launch_overlap<2, F32>, &c, 3);
  printf("  %s products: vector work alone %.3f ms, products alone %.3f ms; half the wavefronts each: %.3f ms "
         "(perfect overlap %.3f, none %.3f)\n", F32 ? "fp32 16x16x4 " : "bf16 16x16x32", v, m, h, (v > m ? v : m) / 2, (v + m) / 2);
}

// ------------------------------------------------------------------ first Hadamard factor: vector form against matrix-core form
// One trip = one worker's share of a wavefront in the fused bf16 kernel for 2^16 blocks: 32 packed registers (64 raw
// entries a lane: four tiles of 16) in, 32 fp32 out, transformed over the 2 bits across the tiles and 3 bits inside.
// The inputs stay in registers (no memory in the loop), so this is the arithmetic alone.
template <bool MATRIX>
__global__ __launch_bounds__(1024) void mb_front(float* out, int iters, unsigned long long m0, uint32_t sign_bytes_lo,
                                                 uint32_t sign_bytes_hi) {
  uint32_t p[32];
  for (int i = 0; i < 32; ++i) p[i] = 0x3F803F80u + (threadIdx.x << 8) + i;
  float acc[32];
  for (int i = 0; i < 32; ++i) acc[i] = 0.0f;
  for (int it = 0; it < iters; ++it) {
    float o[32];
    if (!MATRIX) {
      float t[4][16];
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const uint32_t w = p[q * 8 + r / 2];
          float x = (r & 1) ? __builtin_bit_cast(float, w & 0xFFFF0000u) : __builtin_bit_cast(float, w << 16);
          asm volatile("v_cndmask_b32_e64 %0, %0, -%0, %1" : "+v"(x) : "s"(m0 + (unsigned long long)(q * 16 + r)));
          t[q][r] = x;
        }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float A = t[0][r] + t[1][r], C = t[2][r] - t[3][r];
        o[r] = A + C;
        o[16 + r] = A - C;
      }
#pragma unroll
      for (int half = 0; half < 32; half += 16)
#pragma unroll
        for (int s = 1; s < 8; s <<= 1)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if ((r & s) == 0) {
              const float x = o[half + r], y = o[half + r + s];
              o[half + r] = x + y;
              o[half + r + s] = x - y;
            }
    } else {
      const bf8 hmat = __builtin_bit_cast(bf8, u4{0x3F803F80u, 0xBF803F80u, 0x3F80BF80u, 0xBF80BF80u ^ (threadIdx.x << 31)});
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const uint32_t byte = ((c < 4 ? sign_bytes_lo : sign_bytes_hi) >> (8 * (c & 3))) & 0xFFu;
        u4 x;
#pragma unroll
        for (int d = 0; d < 4; ++d) x[d] = p[c * 4 + d] ^ ((byte * (0x40008000u >> (2 * d))) & 0x80008000u);
        const f4 r4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hmat, __builtin_bit_cast(bf8, x), f4{0, 0, 0, 0}, 0, 0, 0);
        o[c * 4] = r4[0]; o[c * 4 + 1] = r4[1]; o[c * 4 + 2] = r4[2]; o[c * 4 + 3] = r4[3];
      }
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      acc[i] += o[i];
      p[i] += 0x00010001u * (uint32_t)(it & 1);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  float s = 0;
  for (int i = 0; i < 32; ++i) s += acc[i];
  out[blockIdx.x * 1024 + threadIdx.x] = s;
}
template <bool MATRIX> static void launch_front(void* c) {
  auto* x = (IssueCtx*)c;
  hipLaunchKernelGGL((mb_front<MATRIX>), dim3(256), dim3(1024), 0, 0, x->out, x->iters, 0x0123456789ABCDEFull, 0xA5C3960Fu, 0x3C5A0FF0u);
}

// ------------------------------------------------------------------ v_dot2c_f32_bf16 as unpack-and-add
__global__ void mb_dot2_exact(const uint32_t* pk, const float* acc, float* out_lo, float* out_hi, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  out_lo[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, pk[i]), __builtin_bit_cast(bf2, 0x00003F80u), acc[i], false);
  out_hi[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, pk[i]), __builtin_bit_cast(bf2, 0x3F800000u), acc[i], false);
}
static void dot2() {
  const int n = 1 << 20;
  std::vector<uint32_t> pk(n);
  std::vector<float> acc(n), lo(n), hi(n);
  srand(3);
  for (int i = 0; i < n; ++i) {   // values of ordinary magnitude (exponents 0x70..0x8F): no infinities, no denormals
    const uint32_t e1 = 0x70u + rand() % 0x20, e2 = 0x70u + rand() % 0x20, e3 = 0x70u + rand() % 0x20;
    pk[i] = ((uint32_t)(rand() & 1) << 31) | (e1 << 23) | ((uint32_t)(rand() & 0x7F) << 16) | ((uint32_t)(rand() & 1) << 15) | (e2 << 7) | (uint32_t)(rand() & 0x7F);
    const uint32_t a = ((uint32_t)(rand() & 1) << 31) | (e3 << 23) | ((uint32_t)rand() & 0x7FFFFFu);
    memcpy(&acc[i], &a, 4);
  }
  uint32_t* dp; float *da, *dl, *dh;
  CK(hipMalloc(&dp, n * 4)); CK(hipMalloc(&da, n * 4)); CK(hipMalloc(&dl, n * 4)); CK(hipMalloc(&dh, n * 4));
  CK(hipMemcpy(dp, pk.data(), n * 4, hipMemcpyHostToDevice)); CK(hipMemcpy(da, acc.data(), n * 4, hipMemcpyHostToDevice));
  hipLaunchKernelGGL(mb_dot2_exact, dim3(n / 256), dim3(256), 0, 0, dp, da, dl, dh, n);
  CK(hipMemcpy(lo.data(), dl, n * 4, hipMemcpyDeviceToHost)); CK(hipMemcpy(hi.data(), dh, n * 4, hipMemcpyDeviceToHost));
  long bad_lo = 0, bad_hi = 0;
  for (int i = 0; i < n; ++i) {
    const uint32_t l = pk[i] << 16, h = pk[i] & 0xFFFF0000u;
    float fl, fh; memcpy(&fl, &l, 4); memcpy(&fh, &h, 4);
    const float wl = acc[i] + fl, wh = acc[i] + fh;
    bad_lo += memcmp(&wl, &lo[i], 4) != 0;
    bad_hi += memcmp(&wh, &hi[i], 4) != 0;
  }
  printf("v_dot2c_f32_bf16(acc, packed pair, (1, 0)) against acc + low half: %ld of %d differ; (0, 1) against acc + high half: %ld differ\n",
         bad_lo, n, bad_hi);
  CK(hipFree(dp)); CK(hipFree(da)); CK(hipFree(dl)); CK(hipFree(dh));
}

// ------------------------------------------------------------------ re-reading a chunk
// workgroup x reads chunks 8x .. 8x+7 (128 KB each), every chunk R times in a row
template <int R, bool SHORTS>
__global__ __launch_bounds__(1024) void mb_reread(const uint32_t* __restrict__ p, uint32_t* out) {
  uint32_t acc = 0;
  for (int i = 0; i < 8; ++i) {
    const uint32_t* q = p + ((size_t)blockIdx.x * 8 + i) * 32768;
    for (int rep = 0; rep < R; ++rep) {
      if (!SHORTS) {
        u4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = *(const u4*)(q + (j * 1024 + threadIdx.x) * 4);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j][0] ^ v[j][1] ^ v[j][2] ^ v[j][3];
      } else {
        const uint16_t* h = (const uint16_t*)q;
        uint32_t v[64];
#pragma unroll
        for (int j = 0; j < 64; ++j) v[j] = h[j * 1024 + threadIdx.x];
#pragma unroll
        for (int j = 0; j < 64; ++j) acc ^= v[j];
      }
      asm volatile("" : "+v"(acc));
    }
  }
  out[blockIdx.x * 1024 + threadIdx.x] = acc;
}
struct RereadCtx { const uint32_t* p; uint32_t* o; };
template <int R, bool SHORTS> static void launch_reread(void* c) {
  auto* x = (RereadCtx*)c;
  hipLaunchKernelGGL((mb_reread<R, SHORTS>), dim3(4096), dim3(1024), 0, 0, x->p, x->o);
}
template <int R, bool SHORTS> static void run_reread(RereadCtx* c) {
  const float ms = time_ms(launch_reread<R, SHORTS>, c, 3);
  printf("  R = %d, %2d-byte loads: %.3f ms for 4 GiB of distinct data: %5.2f TB/s from memory, %5.2f TB/s into the CUs\n", R,
         SHORTS ? 2 : 16, ms, 4.295 / ms, 4.295 * R / ms);
}
static void reread() {
  printf("a workgroup of 1024 lanes reads 8 chunks of 128 KB, every chunk R times in a row:\n");
  RereadCtx c;
  uint32_t *p, *o;
  CK(hipMalloc(&p, (size_t)32768 * 131072)); CK(hipMemset(p, 1, (size_t)32768 * 131072));
  CK(hipMalloc(&o, 4096 * 1024 * 4));
  c.p = p; c.o = o;
  run_reread<1, false>(&c); run_reread<2, false>(&c); run_reread<4, false>(&c);
  run_reread<1, true>(&c); run_reread<2, true>(&c);
  CK(hipFree(p)); CK(hipFree(o));
}

int main(int argc, char** argv) {
  auto want = [&](const char* s) {
    if (argc < 2) return true;
    for (int i = 1; i < argc; ++i) if (!strcmp(argv[i], s)) return true;
    return false;
  };
  float* out;
  CK(hipMalloc(&out, 256 * 1024 * 4));
  if (want("streams")) streams();
  if (want("issue")) issue(out);
  if (want("overlap")) {
    printf("matrix-core work of two wavefronts of a SIMD under vector work of its other two:\n");
    run_overlap<false>(out);
    run_overlap<true>(out);
  }
  if (want("front")) {
    IssueCtx c = {out, 2000};
    const float v = time_ms(launch_front<false>, &c, 3), m = time_ms(launch_front<true>, &c, 3);
    printf("first Hadamard factor of a worker's share of a wavefront (64 bf16 entries a lane -> 32 fp32), four wavefronts per SIMD:\n");
    printf("  vector form (unpack, sign by lane mask, +-1 combination, 3 stages): %7.1f ns per trip per SIMD\n", v * 1e6 / c.iters);
    printf("  matrix-core form (signs by XOR on packed pairs, 8 bf16 products):   %7.1f ns per trip per SIMD\n", m * 1e6 / c.iters);
  }
  if (want("dot2")) dot2();
  if (want("reread")) reread();
  CK(hipFree(out));
  return 0;
}
