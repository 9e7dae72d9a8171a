/* liboptireduce_hip -- the per-node compute path of OptiReduce (arXiv 2310.06993) on one MI355X.
 *
 * The path: a gradient bucket is encoded with a randomized Hadamard transform before it is cut into
 * N shards and sent (Sec. 3.3; Sec. 3 overview); the node that owns shard r averages the r-th shards
 * of all workers over the entries that the bounded transport delivered (Sec. 3.1.1); the aggregated
 * bucket is decoded (Sec. 3.3; Sec. 4: encode before, decode after the reduction).
 *
 * Conventions common to every call
 *   - Every pointer is a DEVICE pointer owned by the caller.  The library allocates nothing, keeps no
 *     state between calls and may be called from several host threads.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call validates its
 *     arguments on the host, enqueues its kernels on that stream and returns; it never synchronises.
 *     Every argument error (status below OR_ERR_HIP) is found before anything is enqueued: no output
 *     is touched.  OR_ERR_HIP reports a launch that the runtime refused; an entry point that enqueues
 *     several kernels may by then have enqueued the earlier ones, so treat its outputs as undefined.
 *   - Vectors are contiguous.  fp32 data is `float`; bf16 data is passed as uint16_t bit patterns.
 *     Data pointers must be 16-byte aligned, mask pointers 4-byte aligned.
 *   - block_log2 = k selects the transform block B = 2^k, OR_MIN_LOG2 <= k <= OR_MAX_LOG2.
 *   - The random diagonal: entry i of the padded vector (i counted from `base_index` for the first
 *     entry passed) is multiplied by -1 iff bit (i mod 128) of Philox4x32-10(counter = (i div 128,
 *     0, 0) as (lo32, hi32, 0, 0), key = (seed lo32, seed hi32)) is set, bits counted from the least
 *     significant bit of output word 0.  Every worker must use the same seed for a bucket.
 *     `base_index` must be a multiple of max(B, 128).
 *   - The Hadamard matrix is in natural (Sylvester) order, H[u][v] = (-1)^popcount(u & v), scaled by
 *     B^(-1/2) on encode and on decode.
 *   - Masks: one row of shard_len/32 uint32 words per worker; bit j of word w is entry 32w + j;
 *     1 = the entry arrived.  The data slot of an entry that did not arrive is never used in
 *     arithmetic and may hold anything (NaN included).
 *   - A length of 0 is valid and does nothing.
 */
#ifndef OPTIREDUCE_H_
#define OPTIREDUCE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int or_status;
enum {
  OR_OK = 0,
  OR_ERR_NULL = 1,      /* a required pointer is NULL                                          */
  OR_ERR_BLOCK = 2,     /* block_log2 outside [OR_MIN_LOG2, OR_MAX_LOG2]                       */
  OR_ERR_WORKERS = 3,   /* N < 1 or N > OR_MAX_WORKERS                                         */
  OR_ERR_SHAPE = 4,     /* length not a multiple of what the call needs, bad base_index,
                           forbidden overlap, length too large                                */
  OR_ERR_ALIGN = 5,     /* a pointer is not aligned as required                                */
  OR_ERR_WORKSPACE = 6, /* workspace missing or smaller than or_workspace_bytes() says         */
  OR_ERR_HIP = 7        /* a launch failed; or_last_hip_error() gives the hipError_t           */
};

#define OR_MIN_LOG2 5
#define OR_MAX_LOG2 16
#define OR_MAX_WORKERS 255

/* ---- helpers (host only, no GPU work) ------------------------------------------------------- */

/* n rounded up to a whole number of blocks of 2^block_log2 entries (0 if block_log2 is invalid). */
uint64_t or_padded_len(uint64_t n, int block_log2);
/* Bytes of device workspace that or_reduce_decode* / or_fused_path* need for this shard length and
 * block size: 0 for block_log2 <= 14, else 5 bytes per shard entry (rounded up to 256-byte parts).  What
 * the kernels keep there (fp32 sums or means and counts; the shard's sign stream; for the bf16 fused
 * path with block_log2 = 16 what the two workgroups of a block hand to each other, and their flags) is
 * written before it is read within one call: the workspace needs no initialisation, and calls that may
 * overlap in time need workspaces of their own. */
size_t or_workspace_bytes(uint64_t shard_len, int block_log2);
const char* or_status_string(or_status s);
int or_version(void);
/* hipError_t (as int) of the last failed launch on the calling thread, 0 if none. */
int or_last_hip_error(void);

/* Measurement hook (not part of the method).  Arms two caller-created hipEvent_t (either may be NULL)
 * for the NEXT entry-point call made by this thread: `start_event` is attached to the first kernel
 * that call enqueues and receives that kernel's begin timestamp, `stop_event` to the last one and
 * receives its end timestamp (for a call that enqueues several kernels: the first kernel of all and the
 * last of all), so hipEventElapsedTime(start, stop) after a synchronise is the device time of the call
 * without launch gaps.  The arming is consumed by that call whether it succeeds or
 * not; a call that enqueues nothing leaves the events unrecorded. */
or_status or_time_next_call(void* start_event, void* stop_event);

/* ---- Sec. 3.3 encode: out = B^(-1/2) H D grad, blockwise ------------------------------------
 * grad: n entries.  out: or_padded_len(n) entries; the pad of the last block is treated as zeros
 * before the transform.  out == grad is allowed iff n is already a multiple of B; any other overlap
 * is an error.  or_rht_encode is or_rht_encode_at with base_index 0. */
or_status or_rht_encode(const float* grad, uint64_t n, int block_log2, uint64_t seed, float* out, void* stream);
or_status or_rht_encode_at(const float* grad, uint64_t n, int block_log2, uint64_t seed, uint64_t base_index,
                           float* out, void* stream);
/* bf16 gradient in, bf16 encoded out (fp32 arithmetic, one rounding to nearest even at the store). */
or_status or_rht_encode_bf16(const uint16_t* grad, uint64_t n, int block_log2, uint64_t seed, uint64_t base_index,
                             uint16_t* out, void* stream);

/* ---- Sec. 3.1.1 aggregation at the owner of a shard ------------------------------------------
 * shards: [N][shard_len] row-major, row i = worker i's copy of the shard.  masks: [N][shard_len/32].
 * sum_out[e] = sum over workers whose bit e is set (fp32 accumulation, increasing worker index);
 * count_out[e] = how many were set.  shard_len must be a multiple of 32.  Outputs must not overlap
 * the inputs. */
or_status or_masked_reduce(const float* shards, const uint32_t* masks, int N, uint64_t shard_len, float* sum_out,
                           uint8_t* count_out, void* stream);
or_status or_masked_reduce_bf16(const uint16_t* shards, const uint32_t* masks, int N, uint64_t shard_len,
                                float* sum_out, uint8_t* count_out, void* stream);

/* ---- Sec. 3.3 / Sec. 4 decode: out = D B^(-1/2) H agg, first n entries kept -------------------
 * agg: or_padded_len(n) fp32 entries, already the mean.  out: n entries.  In place allowed iff n is
 * a multiple of B. */
or_status or_rht_decode(const float* agg, uint64_t n, int block_log2, uint64_t seed, float* out, void* stream);
or_status or_rht_decode_at(const float* agg, uint64_t n, int block_log2, uint64_t seed, uint64_t base_index,
                           float* out, void* stream);
or_status or_rht_decode_bf16(const float* agg, uint64_t n, int block_log2, uint64_t seed, uint64_t base_index,
                             uint16_t* out, void* stream);

/* ---- fused forms (the calls above chained, with fewer trips through memory) -------------------
 * Counts are identical to those of the chained calls; values agree with them within the tolerance
 * of the path (relative L2 1e-6 for fp32, 1e-2 for bf16): the fused kernels take the mean with a
 * reciprocal and a multiply where or_finalize divides, and sum in their own order.
 * "Averages" (Sec. 3.1.1) is read as sum / number received, 0 where nothing was received.
 *
 * or_finalize_decode: mean = sum / count, then decode.  sum, count: or_padded_len(n) entries. */
or_status or_finalize_decode(const float* sum, const uint8_t* count, uint64_t n, int block_log2, uint64_t seed,
                             uint64_t base_index, float* out, void* stream);
or_status or_finalize_decode_bf16(const float* sum, const uint8_t* count, uint64_t n, int block_log2,
                                  uint64_t seed, uint64_t base_index, uint16_t* out, void* stream);

/* or_reduce_decode: masked aggregation of N encoded shards, mean, decode of that shard.
 * shard_len must be a multiple of B.  out: shard_len entries of the shards' type.  count_out may be
 * NULL.  workspace: device memory of or_workspace_bytes(shard_len, block_log2) bytes, 256-byte
 * aligned, or NULL when that is 0; its contents afterwards are unspecified. */
or_status or_reduce_decode(const float* shards, const uint32_t* masks, int N, uint64_t shard_len, int block_log2,
                           uint64_t seed, uint64_t base_index, float* out, uint8_t* count_out, void* workspace,
                           size_t workspace_bytes, void* stream);
or_status or_reduce_decode_bf16(const uint16_t* shards, const uint32_t* masks, int N, uint64_t shard_len,
                                int block_log2, uint64_t seed, uint64_t base_index, uint16_t* out,
                                uint8_t* count_out, void* workspace, size_t workspace_bytes, void* stream);

/* or_fused_path: the whole path for the shard one node owns, with all N workers' RAW (not yet
 * encoded) slices of that shard resident: encode each slice, keep what arrived, sum and count,
 * mean, decode.  grads: [N][shard_len] raw gradient slices; the encoded value is rounded to the
 * wire type (fp32: no-op; bf16: nearest even) before it is summed, as if it had been stored by
 * or_rht_encode*.  Other arguments as for or_reduce_decode. */
or_status or_fused_path(const float* grads, const uint32_t* masks, int N, uint64_t shard_len, int block_log2,
                        uint64_t seed, uint64_t base_index, float* out, uint8_t* count_out, void* workspace,
                        size_t workspace_bytes, void* stream);
or_status or_fused_path_bf16(const uint16_t* grads, const uint32_t* masks, int N, uint64_t shard_len,
                             int block_log2, uint64_t seed, uint64_t base_index, uint16_t* out, uint8_t* count_out,
                             void* workspace, size_t workspace_bytes, void* stream);

/* or_fused_path_bf16_static: or_fused_path_bf16 for callers that cannot allocate device memory or must not
 * pass a workspace (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
 * The workspace of the kernels for block_log2 > 14 is a static array in device memory inside the library,
 * (5 * OR_STATIC_MAX_SHARD_LEN bytes, 20 MiB, held by every GPU the library runs on until the process ends);
 * for block_log2 <= 14 no workspace is used.  Same arguments, checks, kernels and results as
 * or_fused_path_bf16 otherwise.  block_log2 > 14 with shard_len > OR_STATIC_MAX_SHARD_LEN is rejected
 * with OR_ERR_WORKSPACE.  The call allocates nothing; its first call on a device looks the array's address
 * up (make that call outside a graph capture).  Every call on a GPU uses that GPU's one array: calls with
 * block_log2 > 14 that may overlap in time on one GPU (different streams, several host threads) race on
 * it -- keep them on one stream or order them with events. */
#define OR_STATIC_MAX_SHARD_LEN 4194304ull
or_status or_fused_path_bf16_static(const uint16_t* grads, const uint32_t* masks, int N, uint64_t shard_len,
                                    int block_log2, uint64_t seed, uint64_t base_index, uint16_t* out,
                                    uint8_t* count_out, void* stream);

/* ---- around the path: transform off, second-stage loss, loss monitoring, two-level aggregation ----
 *
 * or_finalize: the "averages" of Sec. 3.1.1 alone, mean = sum / count and 0 where count is 0 -- with
 * or_masked_reduce this is the path with the Hadamard transform switched off (Sec. 3.2.1 enables it
 * only above 2 % loss).  shard_len a multiple of 32; mean_out == sum is allowed for the fp32 form. */
or_status or_finalize(const float* sum, const uint8_t* count, uint64_t shard_len, float* mean_out, void* stream);
or_status or_finalize_bf16(const float* sum, const uint8_t* count, uint64_t shard_len, uint16_t* mean_out,
                           void* stream);

/* or_received_total: Sec. 3.4 monitors the gradient loss of every AllReduce to skip an update or halt.
 * *total_out (device, 8-byte aligned) = sum of the counts = number of (worker, entry) arrivals; the
 * loss fraction of the shard is 1 - total / (N * shard_len).  Exact integer. */
or_status or_received_total(const uint8_t* count, uint64_t shard_len, uint64_t* total_out, void* stream);

/* or_loss_decision: the safeguard of Sec. 3.4 and the activation rule of Sec. 3.2.1 as host arithmetic (no GPU
 * work, no stream; every pointer here is a HOST pointer).  received_total is what or_received_total wrote,
 * copied back by the caller; loss = 1 - received_total / (N * shard_len).
 *   *action_out: OR_ACT_HALT if loss > policy->halt_loss, else OR_ACT_SKIP if loss > policy->skip_loss,
 *                else OR_ACT_APPLY (the paper leaves the threshold and the choice between skipping the
 *                update and halting to the user: set a threshold above 1 to switch that action off);
 *   *transform_on_out: prev_transform_on, or 1 once loss > policy->transform_on_loss (the paper's 2 %;
 *                OR_DEFAULT_TRANSFORM_ON_LOSS) -- the transform stays on once it has been switched on;
 *   *loss_out (may be NULL): the loss fraction.
 * OR_ERR_SHAPE if received_total > N * shard_len or N * shard_len == 0, OR_ERR_NULL for a missing pointer,
 * OR_ERR_WORKERS for N outside 1..OR_MAX_WORKERS; thresholds must not be NaN (OR_ERR_SHAPE). */
#define OR_DEFAULT_TRANSFORM_ON_LOSS 0.02
enum { OR_ACT_APPLY = 0, OR_ACT_SKIP = 1, OR_ACT_HALT = 2 };
typedef struct or_loss_policy {
  double transform_on_loss; /* switch the Hadamard transform on above this loss */
  double skip_loss;         /* drop this round's update above this loss */
  double halt_loss;         /* stop training above this loss */
} or_loss_policy;
or_status or_loss_decision(uint64_t received_total, int N, uint64_t shard_len, const or_loss_policy* policy,
                           int prev_transform_on, int* action_out, int* transform_on_out, double* loss_out);

/* or_rht_decode_masked: decode after loss in the SECOND stage (Sec. 3.1.1: the owner broadcasts its
 * aggregated shard over the same unreliable transport; Sec. 3.3: the transform spreads what is lost).
 * mask: or_padded_len(n)/32 words, bit layout as for shards; an aggregated entry whose bit is clear
 * never arrived, is never read and counts as zero.  Otherwise as or_rht_decode_at / _bf16. */
or_status or_rht_decode_masked(const float* agg, const uint32_t* mask, uint64_t n, int block_log2, uint64_t seed,
                               uint64_t base_index, float* out, void* stream);
or_status or_rht_decode_masked_bf16(const float* agg, const uint32_t* mask, uint64_t n, int block_log2,
                                    uint64_t seed, uint64_t base_index, uint16_t* out, void* stream);

/* or_masked_reduce_pairs: second level of hierarchical 2D TAR (Sec. 3.1.2, Appendix A): every group
 * has aggregated its members into a partial (sum, count) with or_masked_reduce; the partial
 * aggregates of the G groups that arrived are combined, sums with sums and counts with counts.
 * sums: [G][shard_len] fp32, counts: [G][shard_len] uint8, masks: [G][shard_len/32]; 1 <= G <= 255;
 * the counts of one entry must not add up to more than 255. */
or_status or_masked_reduce_pairs(const float* sums, const uint8_t* counts, const uint32_t* masks, int G,
                                 uint64_t shard_len, float* sum_out, uint8_t* count_out, void* stream);

/* or_fused_path_batched: or_fused_path / or_fused_path_bf16 for several buckets that share N,
 * block_log2 and element type, in as few launches as possible (up to 64 buckets per launch).  A DDP
 * bucket (Sec. 3.1.1 footnote: 25 MB by default) is only about a hundred tiles per shard, far too few
 * to fill the GPU alone.  `buckets` is a HOST array, read before the call returns; the device
 * pointers in it follow the rules of or_fused_path (grads/out are float or bf16 bits per `bf16`).
 * Every bucket is validated before anything is enqueued; no output of one bucket may overlap anything
 * of another bucket (OR_ERR_SHAPE).  Buckets of length 0 are skipped.  For block_log2 > 14 the buckets
 * are run one after the other and `workspace` must cover the largest or_workspace_bytes() among them. */
typedef struct or_bucket {
  const void* grads;      /* [N][shard_len] raw slices                  */
  const uint32_t* masks;  /* [N][shard_len/32]                          */
  void* out;              /* shard_len entries                          */
  uint8_t* count_out;     /* shard_len counts, or NULL                  */
  uint64_t shard_len;
  uint64_t seed;
  uint64_t base_index;
} or_bucket;
or_status or_fused_path_batched(const or_bucket* buckets, int n_buckets, int N, int block_log2, int bf16,
                                void* workspace, size_t workspace_bytes, void* stream);

/* The same with the loss statistic of Sec. 3.4 taken inside the same kernels: totals (device, 8-byte
 * aligned, n_buckets entries, or NULL) receives per bucket the number of (worker, entry) arrivals, the
 * value or_received_total gives for that bucket's counts; totals[j] of an empty bucket is 0.  One
 * bucket is the case n_buckets = 1. */
or_status or_fused_path_batched_monitored(const or_bucket* buckets, int n_buckets, int N, int block_log2, int bf16,
                                          uint64_t* totals, void* workspace, size_t workspace_bytes, void* stream);

/* ---- the separate calls on several buckets (Sec. 3.1.1 footnote: DDP hands over 25 MB buckets; one
 * bucket per launch leaves most of the GPU idle).  Same descriptor scheme, same validation rules.
 *
 * or_reduce_decode_batched: or_reduce_decode / _bf16 per bucket; or_bucket.grads holds the ENCODED
 * shards.  totals as in or_fused_path_batched_monitored (may be NULL). */
or_status or_reduce_decode_batched(const or_bucket* buckets, int n_buckets, int N, int block_log2, int bf16,
                                   uint64_t* totals, void* workspace, size_t workspace_bytes, void* stream);

/* or_masked_reduce_batched: or_masked_reduce / _bf16 per bucket (reads shards, masks; writes sum, count;
 * out, seed and base_index are ignored).
 * or_finalize_decode_batched: or_finalize_decode / _bf16 per bucket (reads sum, count; writes out;
 * shards and masks are ignored); every shard_len must be a whole number of blocks; out == sum is
 * allowed for fp32. */
typedef struct or_stage_bucket {
  const void* shards;     /* [N][shard_len] encoded shards (float or bf16 bits per `bf16`) */
  const uint32_t* masks;  /* [N][shard_len/32]                                            */
  float* sum;             /* shard_len fp32 sums                                          */
  uint8_t* count;         /* shard_len counts                                             */
  void* out;              /* shard_len decoded entries (float or bf16 bits per `bf16`)    */
  uint64_t shard_len;
  uint64_t seed;
  uint64_t base_index;
} or_stage_bucket;
or_status or_masked_reduce_batched(const or_stage_bucket* buckets, int n_buckets, int N, int bf16, void* stream);
or_status or_finalize_decode_batched(const or_stage_bucket* buckets, int n_buckets, int block_log2, int bf16,
                                     void* stream);

#ifdef __cplusplus
}
#endif
#endif /* OPTIREDUCE_H_ */
