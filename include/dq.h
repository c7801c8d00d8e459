/*
 * dq.h -- C ABI of the MI355X (gfx950) hot path of DynamiQ's compressed multi-hop
 * all-reduce (arxiv 2602.08923): first-hop compress, the fused
 * decompress-accumulate-recompress (DAR) hop, decompress(+accumulate), a driver that
 * replays ring / butterfly reduce-scatter hops for N simulated workers inside one
 * GPU's HBM, the same three calls for the OCP-MX comparison codec, and the steps on either
 * side of the main stage (statistics, bit allocation, reorder, restore).
 *
 * Conventions shared by every call
 *   - All data pointers are DEVICE pointers owned by the caller, 16-byte aligned
 *     (per-super-group arrays -- means, indices, statistics, positions -- 4-byte aligned;
 *     DQ_EALIGN otherwise).  Descriptor structs (dq_config, dq_chunk, dq_local, dq_replay_desc
 *     and the arrays they point to) are HOST memory, read during the call only.
 *   - `hip_stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work
 *     and return without synchronising; the library allocates device memory only in
 *     dq_create / dq_replay_create and never per call.
 *   - Errors are return codes only; on any error nothing has been enqueued.  Inputs
 *     must be finite and partial sums must stay below the largest bf16: the library does
 *     not check this, and the result for other inputs is unspecified.  (Addresses in device
 *     memory are computed from the descriptors alone, never from data values; the lookups
 *     in the on-chip tables are indexed by the normalised values and rely on finite inputs.)
 *   - The result of a call is a pure function of (config, chunk descriptor, rank,
 *     input bytes): it does not depend on grid size, batching or call order.
 *
 * Data model (paper Section 5 "configuration", Section 3.5): entries come in groups of
 * 16 sharing a u8 scale and super-groups (SG) of 256 = 16 groups sharing a bf16 scale and
 * a code width of 2, 4 or 8 bits (or 16: raw bf16).  A chunk is a run of SGs in increasing
 * width order (its entries either reordered that way or picked from the original tensor
 * through an index, see dq_local).  Packed chunk layout (structure of arrays, each array 16-byte aligned, SG order):
 *   [2-bit codes, 64 B per SG][4-bit codes, 128 B per SG][8-bit codes, 256 B per SG]
 *   [16-bit values, 512 B per SG: raw bf16, "16 bits corresponds to uncompressed values", Section 3.2]
 *   [group scales, 16 u8 per coded SG][SG scales, one u16 bf16 pattern per coded SG], rounded up
 *   to 16 B (the kernels never write those padding bytes); the coded SGs are those at 2, 4 and
 *   8 bits.  A 16-bit SG has no scales and uses no random numbers: compress rounds to bf16
 *   (nearest even), a DAR hop adds in fp32 and rounds back.
 * Entry k of an SG sits at bit offset k*b of the SG's code block (little-endian);
 * code = sign << (b-1) | level index.
 */
#ifndef DQ_H_
#define DQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dq_ctx dq_ctx;       /* opaque: level tables on the device + PRNG key */
typedef struct dq_replay dq_replay; /* opaque: a prepared hop schedule */

typedef enum { DQ_OK = 0, DQ_EINVAL = 1, DQ_EALIGN = 2, DQ_EUNSUPPORTED = 3, DQ_EHIP = 4 } dq_status;
typedef enum { DQ_F32 = 0, DQ_BF16 = 1 } dq_dtype;
typedef enum { DQ_DYNAMIQ = 0, DQ_MXFP8_E4M3 = 1, DQ_MXFP6_E3M2 = 2, DQ_MXFP4_E2M1 = 3 } dq_codec;
typedef enum { DQ_RING = 0, DQ_BUTTERFLY = 1, DQ_CHAIN = 2 } dq_topology;

typedef struct {
  double g4, g8;      /* 1 + 2*eps^2 of the 4-bit and 8-bit level sets (Section 3.3); the
                         paper does not print eps; 1.3 and 1.02 are this library's defaults */
  uint64_t seed;      /* PRNG seed shared by all workers (Section 2.4) */
  uint32_t round;     /* training round: a new round draws fresh random numbers */
  uint32_t n_workers; /* n of the correlated rounding u_i = (pi_i + gamma_i)/n, 1..8192 */
  uint32_t independent_rounding; /* 0: correlated rounding (Section 3.3).  1: every worker rounds on its own,
                         u = gamma in [0,1): the baseline of Section 2.4, kept for comparisons */
  uint32_t reserved;  /* 0 */
} dq_config;

typedef struct {
  uint64_t first_sg; /* global (post-reorder) index of the chunk's first SG; keys the PRNG */
  uint32_t n_sg[4];  /* SGs at 2, 4, 8 and 16 bits, in this order (16 bits: raw bf16 values) */
} dq_chunk;

/* Build the level tables f(eps, r) of Section 3.3 and upload them.  DQ_EINVAL for a null
 * pointer, n_workers outside 1..8192 or level sets that are not strictly increasing in
 * binary32; DQ_EUNSUPPORTED if a level set is too fine for the kernels' search table. */
dq_status dq_create(const dq_config *cfg, dq_ctx **out);
void dq_destroy(dq_ctx *ctx);
/* Start a new training round (changes the PRNG counter only). */
dq_status dq_set_round(dq_ctx *ctx, uint32_t round);

/* Bytes of the packed form of a chunk (pure; layout above). */
size_t dq_packed_bytes(const dq_chunk *chunk);

/* A worker's own entries as the calls below read them (host struct, read during the call).
 *   data      device, 16-byte aligned, `dtype` entries.
 *   mu        NULL, or one fp32 mean per super-group of the chunk (device, 4-byte aligned, in the
 *             chunk's order).  Section 3.1: every worker subtracts mu_j from each entry of
 *             super-group j before it is quantized; here that is one fp32 subtraction on the widened
 *             entry, done where the entry enters the main stage, for every width (callers pass zero
 *             for the 16-bit super-groups: see dq_reorder_mean).  NULL when `data` is not a
 *             gradient but a buffer of sums whose means are already off.
 *   sg_index  NULL: `data` holds the chunk's super-groups back to back in the chunk's order (a
 *             reordered tensor, Section 3.5).  Else one u32 per super-group of the chunk (device):
 *             super-group j of the chunk is data[256 * sg_index[j] ...], i.e. `data` is the
 *             ORIGINAL tensor and the reorder is done by addressing -- whole super-groups (512 B or
 *             1 KB) are gathered, no reorder pass.  The result is the same bytes either way. */
typedef struct {
  const void *data;
  dq_dtype dtype;
  const float *mu;
  const uint32_t *sg_index;
} dq_local;

/* Leaf node of the aggregation topology (Section 3.4 "Fused kernels", kernel 1 of Section 4):
 * quantize the local chunk (minus its means).  rank: the worker doing the compression
 * (0..n_workers-1).  packed_out: dq_packed_bytes(chunk) bytes. */
dq_status dq_compress(dq_ctx *ctx, const dq_local *local, const dq_chunk *chunk, uint32_t rank, void *packed_out,
                      void *hip_stream);

/* Internal node (kernel 3 of Section 4): decode the received partial sum, add the local
 * slice (minus its means), re-quantize; intermediates never leave registers.  packed_out may
 * alias packed_in. */
dq_status dq_dar_hop(dq_ctx *ctx, const void *packed_in, const dq_local *local, const dq_chunk *chunk, uint32_t rank,
                     void *packed_out, void *hip_stream);

/* Sink of the reduce-scatter, non-last parents of a butterfly node, all-gather receivers
 * (kernels 2 and 4 of Section 4): out = decode(packed_in) [+ (local - mu)].  local_or_null may be
 * NULL; out (fp32, one per entry, the chunk's order) may alias an fp32 local->data without sg_index. */
dq_status dq_decompress(dq_ctx *ctx, const void *packed_in, const dq_local *local_or_null, const dq_chunk *chunk,
                        float *out, void *hip_stream);

/* The sink's decompress with the restore of Section 3.4's last paragraph fused in: super-group j of
 * the chunk is written to out_base + origin[j] * 256 (origin: device, one u32 per super-group of the
 * chunk, distinct values) and, if mu_back_or_null is given, fp32(n_workers * mu_back[j]) is added to
 * each of its entries after the decode (and the local addition): what dq_decompress followed by
 * dq_restore computes, without the pass in between.  local_or_null->data must not be out_base. */
dq_status dq_decompress_restore(dq_ctx *ctx, const void *packed_in, const dq_local *local_or_null, const dq_chunk *chunk,
                                const uint32_t *origin, const float *mu_back_or_null, float *out_base, void *hip_stream);

/* ---- OCP Microscaling comparison codec (blocks of 32, E8M0 shared scale, elements
 * E4M3 / E3M2 / E2M1, round-to-nearest-even, saturating; the formats the paper compares
 * against in Section 5 "Baseline compression schemes").  n_entries must be a multiple of
 * 256.  Packed layout: [element codes: 32 / 24 / 16 B per block][one E8M0 byte per block],
 * each array 16-byte aligned.  MXFP6 packs 4 codes into 3 bytes, little-endian. */
size_t dq_mx_packed_bytes(dq_codec fmt, uint64_t n_entries);
dq_status dq_mx_compress(dq_codec fmt, const void *local, dq_dtype dtype, uint64_t n_entries, void *packed_out,
                         void *hip_stream);
dq_status dq_mx_dar_hop(dq_codec fmt, const void *packed_in, const void *local, dq_dtype dtype, uint64_t n_entries,
                        void *packed_out, void *hip_stream);
dq_status dq_mx_decompress(dq_codec fmt, const void *packed_in, const void *local_or_null, dq_dtype dtype,
                           uint64_t n_entries, float *out, void *hip_stream);

/* ---- Hop replay (Section 3.4 "Reduce-scatter", Appendix B): N simulated workers whose
 * reordered gradients all live in this GPU's HBM; a transfer between workers is a pointer
 * hand-off.  One kernel launch per schedule step covers every (worker, chunk) job of that
 * step.  DQ_RING / DQ_BUTTERFLY: worker_grads[w] holds worker w's n_buckets buckets back to
 * back, each n_sg_bucket SGs (a multiple of n_workers; butterfly needs a power of two);
 * bucket b uses widths n_sg_by_width[4*b..4*b+3] and global SG indices starting at
 * first_sg + b*n_sg_bucket; `out` receives the reduced buckets (the SUM over workers, fp32,
 * same order as the inputs).  DQ_CHAIN: the path of one ring chunk: worker_grads[i] is
 * worker i's slice of that chunk (n_buckets = 1, n_sg_bucket = the chunk's SG count); worker
 * 0 compresses, workers 1..n-2 run DAR, worker n-1 decompresses and adds.
 * codec: DQ_DYNAMIQ or an MX format (then n_sg_by_width is ignored).
 * all_gather = 1 appends Section 3.4's "All-gather": one step in which the sink of every chunk
 * (ring: worker c-1 mod n of chunk c; butterfly: worker c; chain: worker n-1) compresses its fp32
 * sum with its own rank, and one step that decompresses every chunk back into `out`, so that
 * `out` ends as what EVERY worker holds after the all-reduce, the sink included (all workers must
 * end with the same bytes).  The decompression is run once per chunk, not once per receiving
 * worker: the n copies would be identical. */
typedef struct {
  dq_topology topology;
  dq_codec codec;
  dq_dtype dtype;
  uint32_t n_buckets;
  uint64_t n_sg_bucket;
  const uint32_t *n_sg_by_width; /* host, [n_buckets][4]: SGs at 2, 4, 8, 16 bits per bucket */
  uint64_t first_sg;
  uint32_t all_gather; /* 0: reduce-scatter only; 1: append the all-gather phase (see above) */
  const float *mu;     /* device, NULL or [n_buckets][n_sg_bucket] means in reordered order (Section 3.1),
                          the same for every worker: taken off each worker's gradient where it enters a
                          kernel, never off an fp32 buffer of sums; `out` is then the sum of the
                          mean-subtracted entries.  DQ_DYNAMIQ only; must stay valid like scratch. */
  const uint32_t *origin; /* device, NULL or [n_buckets][n_sg_bucket]: origin[p] = the place inside its bucket
                          that reordered super-group p came from (dq_reorder_mean writes it).  Then the last
                          launch of the schedule writes every super-group straight to that place of `out` and
                          adds n_workers * mu back: `out` ends in the ORIGINAL order, unnormalized -- the
                          restore fused into the final decompress.  DQ_DYNAMIQ only. */
  uint32_t inputs_in_original_order; /* 1 (needs origin; ring and butterfly): worker_grads hold the ORIGINAL
                          tensors and every kernel that reads a worker's gradient gathers its super-groups
                          through origin (dq_local.sg_index): no reorder pass at all.  0: reordered inputs. */
  uint32_t n_grads;    /* how many pointers worker_grads holds: must equal the context's n_workers
                          (0: not stated, the array is trusted to hold n_workers pointers) */
} dq_replay_desc;

/* Device scratch the replay needs (job tables, packed messages, fp32 keep-buffers). */
size_t dq_replay_scratch_bytes(const dq_ctx *ctx, const dq_replay_desc *desc);
/* Build the schedule and upload its job tables into `scratch` (synchronous).
 * worker_grads: host array of n_workers device pointers.  scratch and out must stay valid
 * until dq_replay_destroy. */
dq_status dq_replay_create(dq_ctx *ctx, const dq_replay_desc *desc, const void *const *worker_grads, void *scratch,
                           size_t scratch_bytes, float *out, dq_replay **plan);
uint32_t dq_replay_n_steps(const dq_replay *plan);
/* Enqueue every step of the schedule: kernel launches only (no allocation, no memset, no
 * synchronisation unless step_ms is given), so a caller may capture the call in a HIP graph.  step_ms: NULL, or a host array of n_steps floats that
 * receives each step's duration measured with HIP events on `hip_stream` (this variant
 * synchronises the stream before returning). */
dq_status dq_replay_run(dq_replay *plan, float *step_ms, void *hip_stream);
/* Enqueue steps first .. first+count-1 only (so that a caller can bracket a run of hop steps
 * with its own events); running all steps in order is the same as dq_replay_run. */
dq_status dq_replay_run_steps(dq_replay *plan, uint32_t first, uint32_t count, void *hip_stream);
/* Enqueue ONE kernel launch of a step: a butterfly step in which nodes both forward and keep
 * (kind 3 below) is two launches, 0 = the re-encoding one (compress at the first step, DAR after),
 * 1 = the decompress-accumulate into the keep-buffers; every other step is launch 0 alone.  Running a
 * step's launches in order is dq_replay_run_steps(plan, step, 1); a caller uses this to time the DAR
 * launch of such a step on its own.  DQ_EINVAL if the step has no such launch. */
dq_status dq_replay_run_launch(dq_replay *plan, uint32_t step, uint32_t launch, void *hip_stream);
/* Per step: kind (0 compress, 1 DAR, 2 decompress-accumulate, 3 DAR and decompress-accumulate,
 * two launches) and the entries it processes, for throughput accounting. */
dq_status dq_replay_step_info(const dq_replay *plan, uint32_t step, uint32_t *kind, uint64_t *entries_dar,
                              uint64_t *entries_other);
/* DQ_RING / DQ_CHAIN: where the packed message that step `step` writes for chunk `chunk` of bucket
 * `bucket` sits inside scratch, and its size (dq_packed_bytes of that chunk) -- what the worker that ran
 * the step would hand to the transport (Section 3.4: the compressed partial sum sent to the next hop).
 * It stays intact until step + 2 has run (two message sets, written alternately).  DQ_EINVAL for the
 * last step (it writes fp32 sums, not a message) or indices out of range; DQ_EUNSUPPORTED for a
 * butterfly plan. */
dq_status dq_replay_message(const dq_replay *plan, uint32_t step, uint32_t bucket, uint32_t chunk, const void **ptr,
                            size_t *bytes);
void dq_replay_destroy(dq_replay *plan);

/* ---------------------------------------------------------------------------------------
 * Steps before and after the main stage.  Same conventions as above (device pointers, the
 * calls enqueue and return); float and index arrays need 4-byte alignment only, gradient
 * tensors 16.  A "bucket" is a run of n_sg_per_bucket super-groups allocated and reordered
 * on its own; buckets lie back to back in every array.
 */

/* Section 3.1: per super-group j of ONE worker's tensor x (n_sg * 256 entries of dtype),
 * mu_out[j] = mean of its entries and F_out[j] = sum of their squares, accumulated in fp32
 * (16 entries left to right per lane, then a 16-lane butterfly). */
dq_status dq_sg_stats(const void *x, dq_dtype dtype, uint64_t n_sg, float *mu_out, float *F_out, void *hip_stream);

/* Section 3.1 / 3.5: what the statistics all-reduce returns.  mu_all and F_all hold the n
 * workers' statistics row-major [n_workers][n_sg]; every contribution is rounded to bf16
 * (nearest even: each worker sends two BF16 numbers per super-group), summed in rank order in
 * fp32; mu[j] = sum / n (one division), F[j] = sum. */
dq_status dq_stats_combine(const float *mu_all, const float *F_all, uint32_t n_workers, uint64_t n_sg, float *mu,
                           float *F, void *hip_stream);

/* Section 3.2 + Appendix A: widths from the summed squared norms F of each bucket (F >= 0;
 * negative values and NaN are unspecified input).  A super-group gets 16 bits if max_width is 16
 * and F >= T816 = T48 * 2^17/257, else 8 bits if F >= T48, else 4 bits if F >= T24 = T48 * 17/512
 * (one fp32 product each: the threshold ratios of Section 3.2), else 2 bits; T48 is the smallest
 * positive fp32 value or +infinity for which sum_j width_j <= max_code_bits (per bucket), found
 * by bisection on the bit pattern.  max_width: 8 (W = {2,4,8}, the paper's prototype) or 16
 * (W = {2,4,8,16}, its large-scale simulation).  DQ_EINVAL if max_code_bits < 2 * n_sg_per_bucket.
 * Outputs per bucket:
 *   widths[j]  the width of super-group j
 *   pos[j]     its index inside the reordered bucket: all 2-bit super-groups first, then the
 *              4-bit, 8-bit and 16-bit ones, each class in original order (Section 3.5)
 *   counts[5b .. 5b+4] = {#2-bit, #4-bit, #8-bit, #16-bit, bit pattern of T48} of bucket b
 * The search runs in one thread block per bucket; for buckets of up to 65,536 super-groups the widths
 * and positions are written by a second launch spread over the GPU. */
dq_status dq_allocate(const float *F, uint32_t n_sg_per_bucket, uint32_t n_buckets, uint64_t max_code_bits,
                      uint32_t max_width, uint8_t *widths, uint32_t *pos, uint32_t *counts, void *hip_stream);

/* Section 3.5: out[super-group pos[j] of the bucket] = x[super-group j]: whole super-groups
 * copied into increasing-width order.  out must not overlap x.  At most 2^24 super-groups per
 * bucket and 65535 buckets (DQ_EUNSUPPORTED beyond). */
dq_status dq_reorder(const void *x, dq_dtype dtype, const uint32_t *pos, uint32_t n_sg_per_bucket, uint32_t n_buckets,
                     void *out, void *hip_stream);

/* Section 3.1: the means the main stage subtracts, in its (reordered) order:
 * mu_main[pos[j]] = mu[j], except that the 16-bit super-groups of a bucket -- its last
 * counts[5b + 3] places, `counts` being what dq_allocate wrote -- get zero: a value sent as raw
 * bf16 gains nothing from the subtraction, and rounding x - mu back to bf16 would make all
 * workers err the same way.  counts_or_null NULL: no 16-bit class.  mu_main must not be mu.
 * origin_or_null, if given, receives the inverse of the positions, origin[pos[j]] = j (per bucket):
 * what dq_decompress_restore and dq_replay_desc.origin take.  Either output may be NULL, not both;
 * without mu_main, mu is not read. */
dq_status dq_reorder_mean(const float *mu_or_null, const uint32_t *pos, const uint32_t *counts_or_null,
                          uint32_t n_sg_per_bucket, uint32_t n_buckets, float *mu_main_or_null,
                          uint32_t *origin_or_null, void *hip_stream);

/* Section 3.4, last paragraph: out[super-group j] = sum[super-group pos[j]] + n_workers *
 * mu_main[pos[j]] (fp32: one product per super-group, one addition per entry; `sum` is the main
 * stage's result in reordered order, a sum over the workers of mean-subtracted entries, mu_main
 * what dq_reorder_mean wrote).  mu_main_or_null NULL: only the permutation is undone. */
dq_status dq_restore(const float *sum, const uint32_t *pos, const float *mu_main_or_null, uint32_t n_workers,
                     uint32_t n_sg_per_bucket, uint32_t n_buckets, float *out, void *hip_stream);

/* ---- Block-wise pipelining (Section 4, "RDMA engine": as soon as a gradient block completes its
 * decompress-accumulate-recompress, its transfer begins while subsequent blocks are processed).
 * One hop of one chunk, cut every block_sg super-groups; on the wire each block is a packed chunk
 * of its own (first_sg advanced, widths as they fall), the blocks back to back, each starting
 * at a multiple of 256 bytes: dq_pipelined_wire_bytes in all.  Block i is (re-)encoded into half
 * i mod 2 of `stage` (dq_pipelined_stage_bytes, two blocks) and copied from there to its place in
 * wire_out -- a device-to-device copy standing in for the network, which also writes the block's
 * padding bytes as zero -- both on stream i mod 2 of the two streams given (compute_stream takes
 * the even blocks, copy_stream the odd ones): the order inside a stream protects a half until it
 * has left, and the encoding of block i+1 overlaps the transfer of block i with two runtime calls
 * per block and no event.  wire_in NULL: the first hop (compress).  `local` describes the whole
 * chunk (means and indices per super-group of the whole chunk).  The two streams must differ;
 * copy_stream is first made to wait for what compute_stream holds at the call (the inputs), and
 * when the call returns compute_stream has been made to wait for copy_stream, so synchronising
 * compute_stream is enough.  The two events of that fork and join belong to the context (made
 * in dq_create): one pipelined call at a time per context.  The bytes of wire_out between the
 * blocks (up to the next multiple of 256) are not written. */
size_t dq_pipelined_wire_bytes(const dq_chunk *chunk, uint32_t block_sg);
size_t dq_pipelined_stage_bytes(const dq_chunk *chunk, uint32_t block_sg);
dq_status dq_dar_hop_pipelined(dq_ctx *ctx, const void *wire_in, const dq_local *local, const dq_chunk *chunk,
                               uint32_t rank, uint32_t block_sg, void *stage, void *wire_out, void *compute_stream,
                               void *copy_stream);

/* The same hop for callers that cannot allocate device memory and have no staging buffer to hand over
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the two-block
 * stage is a static device array inside the library, DQ_STATIC_STAGE_BYTES per GPU, held until the
 * process ends; its address on the context's GPU is looked up in dq_create.  The call allocates
 * nothing and creates nothing (the pipeline's events are made in dq_create); results are those of
 * dq_dar_hop_pipelined byte for byte.  DQ_EUNSUPPORTED (text in dq_last_hip_error) if
 * dq_pipelined_stage_bytes(chunk, block_sg) exceeds DQ_STATIC_STAGE_BYTES; DQ_EINVAL if the context's
 * device is not the current one.  Every call on a GPU shares that GPU's one array: calls that overlap
 * in time on one GPU (other streams, other contexts, other threads) race on it. */
#define DQ_STATIC_STAGE_BYTES (8u << 20)
dq_status dq_dar_hop_pipelined_static(dq_ctx *ctx, const void *wire_in, const dq_local *local, const dq_chunk *chunk,
                                      uint32_t rank, uint32_t block_sg, void *wire_out, void *compute_stream,
                                      void *copy_stream);

/* ---- Measurement aid, not part of the method: a streaming kernel that reads in_bytes and writes
 * out_bytes (out[j] = xor of the input's 16-byte words j, j + n_out, j + 2 n_out, ...; both sizes
 * multiples of 16, 0 < out_bytes <= in_bytes, buffers 16-byte aligned and not overlapping).  With
 * the read : write ratio of a DAR hop (packed partial sum and local slice in, packed partial sum
 * out) its rate is the practical ceiling the benchmark sets that hop against. */
dq_status dq_stream_probe(dq_ctx *ctx, const void *in, size_t in_bytes, void *out, size_t out_bytes, void *hip_stream);

const char *dq_status_str(dq_status s);
/* Last HIP error string seen by this library on the calling thread (for DQ_EHIP). */
const char *dq_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DQ_H_ */
