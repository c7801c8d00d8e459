// Internal declarations shared by the HIP translation units of libdq (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "dq.h"

namespace dq {

constexpr int kGroup = 16;        // entries per group (Section 5 "configuration")
constexpr int kSG = 256;          // entries per super-group
constexpr int kGroupsPerSG = 16;
constexpr int kWaveSGs = 4;       // one wave64 = 64 groups = 4 super-groups per tile
constexpr int kBlockThreads = 256;
constexpr int kBlockWaves = kBlockThreads / 64;
constexpr uint32_t kMaxGridRows = 65535;  // documented limit of gridDim.y

// One unit of work: a chunk of one simulated worker.
struct Job {
  const uint8_t *in;   // packed partial sum (DAR, decompress) or nullptr (compress)
  const void *local;   // local slice, may be nullptr for decompress
  const float *mu;     // one mean per super-group of the chunk, taken off the local entries, or nullptr
  const uint32_t *src; // per super-group of the chunk: which super-group of `local` holds its entries
                       // (nullptr: `local` holds the chunk's super-groups in chunk order)
  void *out;           // packed (compress, DAR) or fp32 (decompress)
  const uint32_t *dest; // decompress: per super-group of the chunk, the super-group index in `out` it is written to
                        // (nullptr: the chunk's own order, from out[0])
  const float *back;    // decompress: per super-group, the mean added back n_workers times, or nullptr
  uint64_t first_sg;   // global index of the chunk's first super-group
  uint32_t n_sg[4];    // super-groups at 2, 4, 8 and 16 bits
  uint32_t rank;       // worker doing the compression (feeds the random streams)
};

inline Job make_job(const uint8_t *in, const void *local, const float *mu, void *out, uint64_t first_sg,
                    const uint32_t n_sg[4], uint32_t rank) {
  Job j;
  j.in = in; j.local = local; j.mu = mu; j.src = nullptr; j.out = out; j.dest = nullptr; j.back = nullptr;
  j.first_sg = first_sg;
  for (int w = 0; w < 4; ++w) j.n_sg[w] = n_sg[w];
  j.rank = rank;
  return j;
}

// Table blob (dword offsets).  The tables whose size does not depend on the level sets come
// first, at constant places, so that the kernels address them with immediate offsets; the two
// search tables, whose size follows the level sets, come last.  The kernels take LDS byte address
// 0 for the start of the blob: they use dynamic LDS only, which starts at 0 when a kernel has no
// static LDS (checked once per context, see static_lds_bytes).
constexpr uint32_t kOffRec = 0;        // 128 pairs {bits((1+m/128)/255), bits(255/(1+m/128))}
constexpr uint32_t kOffDec2 = 256;     // 2-bit decode: 256 bytes x 4 signed levels
constexpr uint32_t kOffDec4 = 1280;    // 4-bit decode: 256 bytes x 2 signed levels
constexpr uint32_t kOffTab4 = 1792;    // 8 pairs {T, D}
constexpr uint32_t kOffDec8 = 1808;    // 8-bit decode: 256 signed levels
constexpr uint32_t kOffTab8 = 2064;    // 128 pairs {T, D}
constexpr uint32_t kOffLut4 = 2320;    // search table of the 4-bit set: (2^m + 1) pairs {next level, candidate index}
constexpr int kRanges = 6;             // copy ranges: common, 2-bit, 4-bit fixed, 8-bit fixed, 4-bit search, 8-bit search

// Everything the kernels need besides the job: PRNG key, worker count, table blob.
struct Params {
  const uint32_t *blob;  // device copy of the table blob
  uint32_t blob_dwords;  // multiple of 4
  uint32_t range_lo[kRanges], range_hi[kRanges];  // dword ranges a block copies into LDS (multiples of 4) ...
  uint32_t range_width[kRanges];                  // ... if it meets tiles of this width index (3: always)
  uint32_t off_lut8;     // search table of the 8-bit set (dword offset; its size follows the set)
  float magic[3];        // 2^(23-m): adding it leaves round(x * 2^m) in the low mantissa bits
  uint32_t key0, key1, round;
  uint32_t n_workers;
  uint32_t n_mask;       // n-1 if n is a power of two, else 0xFFFFFFFF (meaning: use %)
  uint32_t perm_bits;    // ceil(log2 n): width of the integers the rounding permutation mixes
  float inv_n, s_n;
};

enum Kind { kCompress = 0, kDar = 1, kDecompress = 2 };

// kernel launchers (dq_kernels.hip); grid_blocks = thread blocks the GPU keeps resident at once
hipError_t launch_one(Kind kind, dq_dtype dtype, bool has_local, const Job &job, const Params &p, uint32_t grid_blocks,
                      hipStream_t stream);
// gather: some job of the batch has a `src` (jobs without one still take the contiguous path)
hipError_t launch_batch(Kind kind, dq_dtype dtype, bool has_local, bool gather, const Job *jobs_dev, uint32_t n_jobs,
                        uint32_t max_tiles_per_job, uint64_t total_tiles, const Params &p, uint32_t grid_blocks,
                        hipStream_t stream);

// 16 zero bytes at a 16-byte aligned device address, written by a kernel
// dst[0..bytes) = src[0..bytes) in 16-byte words (bytes a multiple of 16), except that the bytes from `valid`
// on are written as zero: the copy that stands in for the wire puts a packed block's padding down itself
hipError_t wire_copy(void *dst, const void *src, size_t bytes, size_t valid, hipStream_t stream);

// Largest static LDS size over the codec kernels (must be 0: they address their tables from LDS byte 0)
hipError_t static_lds_bytes(size_t *bytes);

// streaming probe (probe_kernels.hip): reads in_bytes, writes out_bytes (multiples of 16, out <= in)
hipError_t stream_probe(const void *in, size_t in_bytes, void *out, size_t out_bytes, uint32_t n_cu, hipStream_t stream);

// DQ_OK, or DQ_EHIP after recording the error's text for dq_last_hip_error (dq_api.cpp)
dq_status hip_status(hipError_t e);

struct MxJob {
  const uint8_t *in;
  const void *local;
  void *out;
  uint64_t n_entries;
};
hipError_t mx_launch_one(Kind kind, dq_codec fmt, dq_dtype dtype, bool has_local, const MxJob &job, uint32_t n_cu,
                         hipStream_t stream);
hipError_t mx_launch_batch(Kind kind, dq_codec fmt, dq_dtype dtype, bool has_local, const MxJob *jobs_dev,
                           uint32_t n_jobs, uint64_t max_entries_per_job, uint32_t n_cu, hipStream_t stream);

}  // namespace dq

// context internals shared between dq_api.cpp and dq_replay.cpp
struct dq_ctx {
  dq_config cfg;
  dq::Params params;
  uint32_t *blob_dev;
  uint32_t n_cu;
  uint32_t grid_blocks;  // n_cu x blocks per CU (5, or the DQ_BLOCKS_PER_CU environment variable at dq_create)
  int device;
  hipEvent_t pipe_event[2];  // block pipeline: fork (0) and join (1) of its two streams; made and destroyed with the context
  bool have_event[2];        // which of the two exist
  bool have_events;          // both
  void *static_stage;  // this device's copy of the library's static staging array (dq_dar_hop_pipelined_static), or null
};
