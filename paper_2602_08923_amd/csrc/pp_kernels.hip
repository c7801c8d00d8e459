// Steps before and after the main all-reduce stage, for gfx950: per-super-group statistics
// (Section 3.1), their combination over workers with the bf16 exchange format (Sections 3.1,
// 3.5), the bit allocation with tied thresholds (Section 3.2, Appendix A), the reorder into
// increasing width order (Section 3.5), the means the main stage subtracts in that order
// (Section 3.1) and the final restore (Section 3.4, last paragraph).  All of them stream each entry once; the allocation
// works on 4 bytes per super-group.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dq_device.h"

namespace {

constexpr int kSG = 256;
constexpr int kThreads = 256;

__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
template <typename T>
__device__ __forceinline__ T gld(const void *p) {
  return *reinterpret_cast<const __attribute__((address_space(1))) T *>((uintptr_t)p);
}
template <typename T>
__device__ __forceinline__ void gst(void *p, T v) {
  *reinterpret_cast<__attribute__((address_space(1))) T *>((uintptr_t)p) = v;
}

// fp32 -> bf16 pattern, round to nearest, ties to even (finite inputs)
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  const uint32_t b = f2u(f);
  return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// ---------------------------------------------------------------------------------------
// Statistics.  One wave handles 4 super-groups at a time: lane l owns group l (16 entries,
// 32 or 64 consecutive bytes), sums them left to right in fp32 (squares by fma), and the 16
// lanes of a row are combined by a butterfly (partner distance 1, 2, 4, 8).
template <typename LT>
__global__ void __launch_bounds__(kThreads) k_stats(const void *x, uint64_t n_sg, float *mu, float *F) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint64_t wave = (uint64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  const uint64_t n_waves = (uint64_t)gridDim.x * (kThreads / 64);
  const uint64_t n_tiles = (n_sg + 3) / 4;
  for (uint64_t t = wave; t < n_tiles; t += n_waves) {
    const uint64_t sg = min(t * 4 + (lane >> 4), n_sg - 1);  // idle rows redo the last SG, store nothing
    const uint64_t first = sg * kSG + (lane & 15u) * 16;
    float v[16];
    if constexpr (sizeof(LT) == 4) {
      const uint8_t *p = static_cast<const uint8_t *>(x) + first * 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const f32x4 q = gld<f32x4>(p + 16 * i);
        v[4 * i] = q.x; v[4 * i + 1] = q.y; v[4 * i + 2] = q.z; v[4 * i + 3] = q.w;
      }
    } else {
      const uint8_t *p = static_cast<const uint8_t *>(x) + first * 2;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const u32x4 q = gld<u32x4>(p + 16 * i);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          v[8 * i + 2 * j] = u2f(w[j] << 16);
          v[8 * i + 2 * j + 1] = u2f(w[j] & 0xFFFF0000u);
        }
      }
    }
    float s = 0.0f, f = 0.0f;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      s += v[k];
      f = __builtin_fmaf(v[k], v[k], f);
    }
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) {
      s += __shfl_xor(s, d, 64);
      f += __shfl_xor(f, d, 64);
    }
    if ((lane & 15u) == 0 && t * 4 + (lane >> 4) < n_sg) {
      gst<float>(mu + sg, s * (1.0f / kSG));
      gst<float>(F + sg, f);
    }
  }
}

// Combination over workers: contributions rounded to bf16 (what is exchanged), summed in rank
// order in fp32; the mean of the means by one division.
__global__ void __launch_bounds__(kThreads) k_combine(const float *mu_all, const float *F_all, uint32_t n, uint64_t J,
                                                      float *mu, float *F) {
  const uint64_t j = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (j >= J) return;
  float sm = 0.0f, sf = 0.0f;
  for (uint32_t i = 0; i < n; ++i) {
    sm = sm + u2f(bf16_rne(gld<float>(mu_all + (uint64_t)i * J + j)) << 16);
    sf = sf + u2f(bf16_rne(gld<float>(F_all + (uint64_t)i * J + j)) << 16);
  }
  gst<float>(mu + j, sm / (float)n);
  gst<float>(F + j, sf);
}

// ---------------------------------------------------------------------------------------
// Allocation: one block of 1024 threads per bucket.  Super-group j = 1024*k + t sits in slot k
// of thread t (a register when the bucket has at most 64 rows of 1024), so every global access
// is coalesced.  Values are handled as int32 bit patterns: non-negative floats order like their
// patterns, and the difference of two patterns below 2^31 has the sign of the comparison,
// F >= theta  <=>  bits(F) - bits(theta) >= 0.  Negative values and NaN count as +0; slots past
// the bucket's end hold -1, which is below every threshold.
constexpr int kAllocThreads = 1024;
constexpr int kAllocWaves = kAllocThreads / 64;
constexpr int kRegs = 64;
constexpr uint32_t kBins = 2048;  // 2 per thread
constexpr uint32_t kCap = 4096;   // candidates kept per threshold

__device__ __forceinline__ int32_t pattern_of(float f) { return f > 0.0f ? (int32_t)f2u(f) : 0; }

// class 0, 1, 2, 3 = 2, 4, 8, 16 bits; 4 = no super-group.  Section 3.2's tied thresholds:
// p8 = pattern of T_{4,8}, p4 = pattern of T_{2,4} = T_{4,8} * 17/512, p16 = pattern of
// T_{8,16} = T_{4,8} * 2^17/257 (0x7FFFFFFF, above every value, when 16 bits are not allowed).
__device__ __forceinline__ uint32_t class_of(int32_t v, int32_t p4, int32_t p8, int32_t p16) {
  return v < 0 ? 4u : (v >= p16 ? 3u : (v >= p8 ? 2u : (v >= p4 ? 1u : 0u)));
}
constexpr int32_t kNever = 0x7FFFFFFF;
__device__ __forceinline__ int32_t p4_from(uint32_t pattern) { return (int32_t)f2u(u2f(pattern) * (17.0f / 512.0f)); }
__device__ __forceinline__ int32_t p16_from(uint32_t pattern, bool allow16) {
  return allow16 ? (int32_t)f2u(u2f(pattern) * (131072.0f / 257.0f)) : kNever;
}

// ---- the same search spread over the GPU (dq_allocate_wide).  The threshold T_{4,8} is bracketed by
// histograms that many blocks build together: a level takes the bracket (lo, hi) -- lo does not
// fit or is 0, hi fits -- and counts, in kNB bins each, the patterns that can still change the
// number at or above T_{4,8} (those strictly inside (lo, hi)) and the number at or above T_{2,4}
// (those in [p4(lo), p4(hi))).  On a bin boundary t the first number is exact and the second lies
// between two suffix counts, which gives a cost that surely fits and one that surely does not:
// the next, tighter bracket.  Two levels bring a bracket of 2^31 patterns down to about 2^9; one
// block then finishes the bisection over the few patterns left, and a last launch writes the
// positions.  Every block of a level writes its own counts and the next launch adds them up: no
// atomics on global memory, nothing to clear, the same result whatever the grid.
constexpr uint32_t kNB = 2048;                 // bins per level and threshold
constexpr uint32_t kPartWords = 2 * kNB + 2;   // a block's record: 8-bit bins, 4-bit bins, counts at or above hi and p4(hi)
constexpr int kLevelThreads = 1024;
constexpr uint32_t kMaxLevelBlocks = 8;        // blocks per bucket and level: that many records are added up per bin
constexpr uint32_t kInfPattern = 0x7F800000u;

struct Ranges {
  uint32_t lo, hi, lo4, hi4;  // patterns; bins: (v - lo) >> s8 for lo < v < hi, (v - lo4) >> s4 for lo4 <= v < hi4
  uint32_t s8, s4;
};
__device__ __forceinline__ uint32_t p4_pattern(uint32_t pattern) { return f2u(u2f(pattern) * (17.0f / 512.0f)); }
__device__ __forceinline__ uint32_t shift_for(uint32_t span) {  // smallest s with (span - 1) >> s below kNB
  uint32_t s = 0;
  while (((span - 1) >> s) >= kNB) ++s;
  return s;
}
__device__ __forceinline__ Ranges ranges_of(uint32_t lo, uint32_t hi) {
  Ranges r;
  r.lo = lo; r.hi = hi; r.lo4 = p4_pattern(lo); r.hi4 = p4_pattern(hi);
  r.s8 = hi > lo ? shift_for(hi - lo) : 0u;
  r.s4 = r.hi4 > r.lo4 ? shift_for(r.hi4 - r.lo4) : 0u;
  return r;
}

// h[0..kNB) bin counts in LDS -> suffix counts h[i] = members of bins i and above, h[kNB] = h[kNB+1] = 0.
// Thread t of T owns kNB / T consecutive bins; `wsum` has T / 64 words.  Ends with a barrier.
template <int T>
__device__ __forceinline__ void to_suffix(uint32_t *h, uint32_t *wsum, uint32_t tid) {
  constexpr int kPer = kNB / T;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  uint32_t v[kPer], sum = 0;
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    v[k] = h[tid * kPer + k];
    sum += v[k];
  }
  uint32_t inc = sum;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = __shfl_up(inc, d, 64);
    if (lane >= (uint32_t)d) inc += up;
  }
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < T / 64; ++w) {
    const uint32_t t = wsum[w];
    before += (uint32_t)w < wave ? t : 0u;
    all += t;
  }
  uint32_t s = all - (before + inc - sum);  // members of this thread's first bin and above
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    h[tid * kPer + k] = s;
    s -= v[k];
  }
  if (tid == 0) h[kNB] = h[kNB + 1] = 0;
  __syncthreads();
}

// A level's records (G blocks of kPartWords words) added up into LDS: h8, h4 (kNB + 2 words each) and
// base[0..1] = patterns at or above hi and p4(hi); then suffix counts, then the tighter bracket.
// `ext`: two more LDS words.  Every thread of the block returns the same (lo, hi).
template <int T>
__device__ __forceinline__ void next_bracket(const uint32_t *part, uint32_t G, const Ranges &R, uint32_t J,
                                             uint64_t max_code_bits, uint32_t *h8, uint32_t *h4, uint32_t *base,
                                             uint32_t *wsum, uint32_t *ext, uint32_t tid, uint32_t &lo, uint32_t &hi) {
  // five rounds of loads (40 per thread) are requested before the first is used: the sum is
  // bound by latency, not by the 0.13 MB it reads
  constexpr uint32_t kRounds = (kPartWords + T - 1) / T, kAhead = 5;
#pragma unroll
  for (uint32_t r0 = 0; r0 < kRounds; r0 += kAhead) {
    uint32_t v[kAhead][kMaxLevelBlocks];
#pragma unroll
    for (uint32_t r = 0; r < kAhead; ++r) {
      const uint32_t i = min((r0 + r) * T + tid, kPartWords - 1);
#pragma unroll
      for (uint32_t g = 0; g < kMaxLevelBlocks; ++g) v[r][g] = gld<uint32_t>(part + (uint64_t)min(g, G - 1) * kPartWords + i);
    }
#pragma unroll
    for (uint32_t r = 0; r < kAhead; ++r) {
      const uint32_t i = (r0 + r) * T + tid;
      uint32_t s = 0;
#pragma unroll
      for (uint32_t g = 0; g < kMaxLevelBlocks; ++g) s += g < G ? v[r][g] : 0u;
      if (i < kNB) h8[i] = s;
      else if (i < 2 * kNB) h4[i - kNB] = s;
      else if (i < kPartWords) base[i - 2 * kNB] = s;
    }
  }
  __syncthreads();
  to_suffix<T>(h8, wsum, tid);
  to_suffix<T>(h4, wsum, tid);
  lo = R.lo;
  hi = R.hi;
  if (R.hi - R.lo <= 1) return;
  const uint32_t base8 = base[0], base4 = base[1];
  // thresholds on bin boundaries inside the bracket: t_i = lo + (i << s8), i = 1..m
  const uint32_t m = (R.hi - R.lo - 1) >> R.s8;
  auto cost_bounds = [&](uint32_t i, uint64_t &c_min, uint64_t &c_max) {
    const uint64_t fixed = 2ull * J + 4ull * (base8 + h8[i]);
    const uint32_t q = p4_pattern(R.lo + (i << R.s8));  // not below lo4: the product is monotone
    uint32_t a_min = 0, a_max = 0;
    if (q < R.hi4) {
      const uint32_t i4 = (q - R.lo4) >> R.s4;
      a_min = h4[i4 + 1];
      a_max = h4[i4];
    }
    c_min = fixed + 2ull * (base4 + a_min);
    c_max = fixed + 2ull * (base4 + a_max);
  };
  // every boundary is tried at once (a bisection would be twenty dependent LDS round trips): the
  // smallest that surely fits and the largest that surely does not; index 0 stands for lo, m + 1 for hi
  if (tid == 0) {
    ext[0] = m + 1;
    ext[1] = 0;
  }
  __syncthreads();
  uint32_t fit = m + 1, no = 0;
  for (uint32_t i = tid + 1; i <= m; i += T) {
    uint64_t c_min, c_max;
    cost_bounds(i, c_min, c_max);
    if (c_max <= max_code_bits) fit = min(fit, i);
    if (c_min > max_code_bits) no = max(no, i);
  }
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    fit = min(fit, (uint32_t)__shfl_xor(fit, d, 64));
    no = max(no, (uint32_t)__shfl_xor(no, d, 64));
  }
  if ((tid & 63u) == 0) {
    atomicMin(&ext[0], fit);
    atomicMax(&ext[1], no);
  }
  __syncthreads();
  fit = ext[0];
  no = ext[1];
  if (fit <= m) hi = R.lo + (fit << R.s8);
  if (no >= 1) lo = R.lo + (no << R.s8);
}

// One level: grid (G, buckets).  FIRST counts inside the widest bracket, (0, +infinity); the
// second level first reads the first level's records and tightens the bracket, which block 0 of
// the bucket also leaves in ctl[0..1] for the kernel that finishes the search.
template <bool FIRST>
__global__ void __launch_bounds__(kLevelThreads) k_alloc_level(const float *F_all, uint32_t J, uint64_t max_code_bits,
                                                               const uint32_t *part_in_all, uint32_t *part_out_all,
                                                               uint32_t *ctl_all) {
  __shared__ uint32_t h8[kNB + 2], h4[kNB + 2];
  __shared__ uint32_t wsum[kLevelThreads / 64], base[2], red[2][kLevelThreads / 64];
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t G = gridDim.x, bucket = blockIdx.y;
  const float *F = F_all + (uint64_t)bucket * J;
  Ranges R = ranges_of(0u, kInfPattern);
  if constexpr (!FIRST) {
    uint32_t lo, hi;
    next_bracket<kLevelThreads>(part_in_all + (uint64_t)bucket * G * kPartWords, G, R, J, max_code_bits, h8, h4, base,
                                wsum, &red[0][0], tid, lo, hi);
    R = ranges_of(lo, hi);
    if (blockIdx.x == 0 && tid == 0) {
      gst<uint32_t>(ctl_all + 4ull * bucket, lo);
      gst<uint32_t>(ctl_all + 4ull * bucket + 1, hi);
    }
    __syncthreads();  // h8 and h4 are cleared next
  }
  for (uint32_t i = tid; i < kNB; i += kLevelThreads) h8[i] = h4[i] = 0;
  __syncthreads();
  const uint32_t per = (J + G - 1) / G;
  const uint32_t j0 = min(J, blockIdx.x * per), j1 = min(J, j0 + per);
  uint32_t a8 = 0, a4 = 0;
  for (uint32_t j = j0 + tid; j < j1; j += kLevelThreads) {
    const uint32_t v = (uint32_t)pattern_of(gld<float>(F + j));
    if (v > R.lo && v < R.hi) atomicAdd(&h8[(v - R.lo) >> R.s8], 1u);
    if (v >= R.lo4 && v < R.hi4) atomicAdd(&h4[(v - R.lo4) >> R.s4], 1u);
    a8 += v >= R.hi ? 1u : 0u;
    a4 += v >= R.hi4 ? 1u : 0u;
  }
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    a8 += __shfl_xor(a8, d, 64);
    a4 += __shfl_xor(a4, d, 64);
  }
  if (lane == 0) {
    red[0][wave] = a8;
    red[1][wave] = a4;
  }
  __syncthreads();
  uint32_t *out = part_out_all + ((uint64_t)bucket * G + blockIdx.x) * kPartWords;
  for (uint32_t i = tid; i < kNB; i += kLevelThreads) {
    gst<uint32_t>(out + i, h8[i]);
    gst<uint32_t>(out + kNB + i, h4[i]);
  }
  if (tid < 2) {
    uint32_t s = 0;
#pragma unroll
    for (int w = 0; w < kLevelThreads / 64; ++w) s += red[tid][w];
    gst<uint32_t>(out + 2 * kNB + tid, s);
  }
}

// Widths and positions once the threshold is known (counts[5b..5b+4] as the search left them):
// grid (ceil(J / 1024), buckets).  A block first counts the members of each class among the
// super-groups before its own 1024 (at most 64 rounds for the sizes this path takes), then ranks
// its own: position = first place of the class + members before the block + members in earlier
// waves + members in lower lanes.
__global__ void __launch_bounds__(kAllocThreads) k_alloc_positions(const float *F_all, uint32_t J, const uint32_t *counts_all,
                                                                   uint8_t *widths_all, uint32_t *pos_all) {
  __shared__ uint32_t before[kAllocWaves][3], mine_w[kAllocWaves][3];
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint64_t first = (uint64_t)blockIdx.y * J;
  const float *F = F_all + first;
  const uint32_t *cnt = counts_all + 5ull * blockIdx.y;
  const int32_t p8 = (int32_t)gld<uint32_t>(cnt + 4), p4 = p4_from((uint32_t)p8);
  const uint32_t n0 = gld<uint32_t>(cnt), n1 = gld<uint32_t>(cnt + 1);
  const uint32_t start[3] = {0u, n0, n0 + n1};
  uint32_t c[3] = {0u, 0u, 0u};
  constexpr uint32_t kAhead = 32;  // rows of 1024 before this block, that many loads in flight
  for (uint32_t r0 = 0; r0 < blockIdx.x; r0 += kAhead) {
    float f[kAhead];
#pragma unroll
    for (uint32_t r = 0; r < kAhead; ++r) f[r] = gld<float>(F + min(r0 + r, blockIdx.x - 1) * kAllocThreads + tid);
#pragma unroll
    for (uint32_t r = 0; r < kAhead; ++r) {
      const uint32_t k = r0 + r < blockIdx.x ? class_of(pattern_of(f[r]), p4, p8, kNever) : 4u;
      c[0] += k == 0 ? 1u : 0u;
      c[1] += k == 1 ? 1u : 0u;
      c[2] += k == 2 ? 1u : 0u;
    }
  }
  const uint32_t j = blockIdx.x * kAllocThreads + tid;
  const uint32_t k = j < J ? class_of(pattern_of(gld<float>(F + j)), p4, p8, kNever) : 4u;
  const uint64_t b0 = __ballot(k == 0), b1 = __ballot(k == 1), b2 = __ballot(k == 2);
#pragma unroll
  for (int i = 0; i < 3; ++i) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) c[i] += __shfl_xor(c[i], d, 64);
  }
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < 3; ++i) before[wave][i] = c[i];
    mine_w[wave][0] = (uint32_t)__builtin_popcountll(b0);
    mine_w[wave][1] = (uint32_t)__builtin_popcountll(b1);
    mine_w[wave][2] = (uint32_t)__builtin_popcountll(b2);
  }
  __syncthreads();
  if (k < 3) {
    uint32_t at = start[k];
#pragma unroll
    for (int w = 0; w < kAllocWaves; ++w) at += before[w][k] + ((uint32_t)w < wave ? mine_w[w][k] : 0u);
    const uint64_t mine = k == 0 ? b0 : (k == 1 ? b1 : b2);
    at += __builtin_amdgcn_mbcnt_hi((uint32_t)(mine >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mine, 0u));
    gst<uint8_t>(widths_all + first + j, (uint8_t)(2u << k));
    gst<uint32_t>(pos_all + first + j, at);
  }
}

// WIDE: the bracket comes from the two histogram levels (their second level's records and
// ctl[0..1]), the kernel ends once counts[5b..5b+4] are written, positions are another launch.
template <bool IN_REGS, bool WIDE = false>
__global__ void __launch_bounds__(kAllocThreads) k_allocate(const float *F_all, uint32_t J, uint64_t max_code_bits,
                                                            bool allow16, uint8_t *widths_all, uint32_t *pos_all,
                                                            uint32_t *counts_all, const uint32_t *part_all = nullptr,
                                                            uint32_t n_part = 0, const uint32_t *ctl_all = nullptr) {
  static_assert(!WIDE || IN_REGS, "the wide search keeps the bucket in registers");
  __shared__ uint32_t red[2][3][kAllocWaves];
  __shared__ uint32_t tot[kRegs * kAllocWaves][4];  // per (row, wave): class counts, then their exclusive scan
  __shared__ uint32_t wsum[kAllocWaves][4];
  __shared__ uint32_t hist[kBins + 2];   // top-11-bit histogram, then suffix counts (register path)
  __shared__ int32_t cand[2][kCap];      // patterns that can still change c8 / c4
  __shared__ uint32_t ncand[2];
  const float *F = F_all + (uint64_t)blockIdx.x * J;
  uint8_t *widths = widths_all + (uint64_t)blockIdx.x * J;
  uint32_t *pos = pos_all + (uint64_t)blockIdx.x * J;
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t rows = (J + kAllocThreads - 1) / kAllocThreads;
  int32_t fr[IN_REGS ? kRegs : 1];
  if constexpr (IN_REGS) {
#pragma unroll
    for (int k = 0; k < kRegs; ++k) {
      const uint32_t j = k * kAllocThreads + tid;  // all loads in flight at once: clamp, then mask
      const int32_t v = pattern_of(gld<float>(F + min(j, J - 1)));
      fr[k] = j < J ? v : -1;
    }
  }
  // Counts over the wave of super-groups at or above T_{2,4} and T_{4,8}.  In registers a funnel
  // shift collects the sign bits of 32 differences in a word and one population count per word
  // turns them into the number below the threshold.
  auto count = [&](int32_t p4, int32_t p8, int32_t p16, uint32_t &c4, uint32_t &c8, uint32_t &c16) {
    uint32_t a4 = 0, a8 = 0, a16 = 0;
    if constexpr (IN_REGS) {
      uint32_t below4 = 0, below8 = 0, below16 = 0;
#pragma unroll
      for (int h = 0; h < kRegs / 32; ++h) {
        uint32_t m4 = 0, m8 = 0;
#pragma unroll
        for (int k = 0; k < 32; ++k) {
          m4 = __builtin_amdgcn_alignbit(m4, (uint32_t)(fr[32 * h + k] - p4), 31);
          m8 = __builtin_amdgcn_alignbit(m8, (uint32_t)(fr[32 * h + k] - p8), 31);
        }
        below4 += __builtin_popcount(m4);
        below8 += __builtin_popcount(m8);
        if (allow16) {
          uint32_t m16 = 0;
#pragma unroll
          for (int k = 0; k < 32; ++k) m16 = __builtin_amdgcn_alignbit(m16, (uint32_t)(fr[32 * h + k] - p16), 31);
          below16 += __builtin_popcount(m16);
        } else {
          below16 += 32;
        }
      }
      a4 = kRegs - below4;
      a8 = kRegs - below8;
      a16 = kRegs - below16;
    } else {
      for (uint32_t j = tid; j < J; j += kAllocThreads) {
        const int32_t v = pattern_of(gld<float>(F + j));
        a4 += v >= p4 ? 1u : 0u;
        a8 += v >= p8 ? 1u : 0u;
        a16 += v >= p16 ? 1u : 0u;
      }
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      a4 += __shfl_xor(a4, d, 64);
      a8 += __shfl_xor(a8, d, 64);
      a16 += __shfl_xor(a16, d, 64);
    }
    c4 = a4; c8 = a8; c16 = a16;
  };
  // The waves' counts meet in LDS, in one of two buffers by turns, so that one barrier per round
  // is enough: a wave can only be one round ahead of the slowest reader.
  uint32_t turn = 0;
  auto block_counts = [&](uint32_t pattern, uint32_t &s4, uint32_t &s8, uint32_t &s16) {
    uint32_t c4, c8, c16;
    count(p4_from(pattern), (int32_t)pattern, p16_from(pattern, allow16), c4, c8, c16);
    if (lane == 0) {
      red[turn][0][wave] = c4;
      red[turn][1][wave] = c8;
      red[turn][2][wave] = c16;
    }
    __syncthreads();
    s4 = 0; s8 = 0; s16 = 0;
#pragma unroll
    for (int w = 0; w < kAllocWaves; ++w) {
      s4 += red[turn][0][w];
      s8 += red[turn][1][w];
      s16 += red[turn][2][w];
    }
    turn ^= 1u;
  };
  // Wanted: the smallest fp32 pattern in [1, +inf] whose allocation fits (the host has checked
  // 2J <= budget).  An SG at or above T_{4,8} is also at or above T_{2,4}, so
  // cost = 2J + 2*c4 + 4*c8, which never increases with the threshold: bisection from any
  // bracket (lo does not fit or is 0, hi fits) ends at the same pattern.
  auto p4_of = [](uint32_t pattern) { return f2u(u2f(pattern) * (17.0f / 512.0f)); };
  uint32_t lo = 0, hi = 0x7F800000u;
  bool narrowed = false;
  uint32_t base4 = 0, base8 = 0;
  if constexpr (IN_REGS) {
  if (!allow16) {  // with a third threshold in play everything is counted every round
    uint32_t b_fit = 0;
    if constexpr (WIDE) {
      // the 4-bit bins share the memory of `tot`, which only the positions use
      uint32_t *h4 = &tot[0][0];
      static_assert(sizeof(tot) >= (kNB + 2) * sizeof(uint32_t) && kBins == kNB, "bins of the wide search");
      const uint32_t *ctl = ctl_all + 4ull * blockIdx.x;
      const Ranges R = ranges_of(gld<uint32_t>(ctl), gld<uint32_t>(ctl + 1));
      next_bracket<kAllocThreads>(part_all + (uint64_t)blockIdx.x * n_part * kPartWords, n_part, R, J, max_code_bits, hist,
                                  h4, ncand, &wsum[0][0], &red[0][0][0], tid, lo, hi);
      __syncthreads();  // ncand (the two base counts) is cleared below
    } else {
    // (1) Histogram of the patterns' top 11 bits (bin b = patterns [b << 20, (b+1) << 20);
    //     2040 << 20 is +infinity), turned into suffix counts S[b] = #{v : bin(v) >= b}.
    for (uint32_t b = tid; b < kBins + 2; b += kAllocThreads) hist[b] = 0;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kRegs; ++k)
      if (fr[k] >= 0) atomicAdd(&hist[(uint32_t)fr[k] >> 20], 1u);
    __syncthreads();
    {
      // thread t owns bins 2t and 2t+1; suffix scan = total - exclusive prefix
      const uint32_t h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
      uint32_t inc = h0 + h1;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = __shfl_up(inc, d, 64);
        if (lane >= (uint32_t)d) inc += up;
      }
      if (lane == 63) wsum[wave][0] = inc;
      __syncthreads();
      uint32_t before = 0, all = 0;
#pragma unroll
      for (int w = 0; w < kAllocWaves; ++w) {
        const uint32_t t = wsum[w][0];
        before += (uint32_t)w < wave ? t : 0u;
        all += t;
      }
      const uint32_t excl = before + inc - (h0 + h1);  // patterns in bins below 2t
      hist[2 * tid] = all - excl;
      hist[2 * tid + 1] = all - excl - h0;
      if (tid == 0) hist[kBins] = hist[kBins + 1] = 0;
      __syncthreads();
    }
    // (2) Bracket in whole bins, by every thread alike (LDS reads only).  For a threshold on a
    //     bin boundary c8 = S[b] is exact and c4 lies in [S[bin4 + 1], S[bin4]], bin4 the bin of
    //     T_{2,4}: an upper and a lower bound of the cost, both monotone.
    auto cost_bounds = [&](uint32_t b, uint64_t &c_min, uint64_t &c_max) {
      const uint32_t bin4 = p4_of(b << 20) >> 20;
      const uint64_t fixed = 2ull * J + 4ull * hist[b];
      c_min = fixed + 2ull * hist[bin4 + 1];
      c_max = fixed + 2ull * hist[bin4];
    };
    uint32_t b_no = 0;
    b_fit = kBins - 8;  // 2040: +infinity, everything at 2 bits
    while (b_fit - b_no > 1) {             // smallest bin boundary that surely fits
      const uint32_t mid = b_no + (b_fit - b_no) / 2;
      uint64_t c_min, c_max;
      cost_bounds(mid, c_min, c_max);
      if (c_max <= max_code_bits) b_fit = mid; else b_no = mid;
    }
    uint32_t b_open = b_fit;
    b_no = 0;                              // pattern 0 is no threshold: "does not fit"
    while (b_open - b_no > 1) {            // largest bin boundary that surely does not fit
      const uint32_t mid = b_no + (b_open - b_no) / 2;
      uint64_t c_min, c_max;
      cost_bounds(mid, c_min, c_max);
      if (c_min > max_code_bits) b_no = mid; else b_open = mid;
    }
    lo = b_no << 20;
    hi = b_fit << 20;
    }
    // (3) Only patterns strictly inside (lo, hi) can change c8 while the threshold moves in
    //     (lo, hi], and only patterns in [p4(lo), p4(hi)) can change c4: collect them in LDS.
    const int32_t lo8 = (int32_t)lo, hi8 = (int32_t)hi, lo4 = (int32_t)p4_of(lo), hi4 = (int32_t)p4_of(hi);
    if (tid < 2) ncand[tid] = 0;
    __syncthreads();
    uint32_t always4 = 0, always8 = 0;
#pragma unroll
    for (int k = 0; k < kRegs; ++k) {
      const int32_t v = fr[k];
      const bool in8 = v > lo8 && v < hi8, in4 = v >= lo4 && v < hi4;
      always4 += v >= hi4 ? 1u : 0u;
      if constexpr (WIDE) always8 += v >= hi8 ? 1u : 0u;
      if constexpr (WIDE) {
        // after two histogram levels a candidate is rare: one LDS atomic each, no wave-wide work
        // (a count already past the capacity is not raised further: the search then counts everything)
        const volatile uint32_t *seen = ncand;
        if (in8 && seen[0] <= kCap) {
          const uint32_t at = atomicAdd(&ncand[0], 1u);
          if (at < kCap) cand[0][at] = v;
        }
        if (in4 && seen[1] <= kCap) {
          const uint32_t at = atomicAdd(&ncand[1], 1u);
          if (at < kCap) cand[1][at] = v;
        }
        continue;
      }
      const uint64_t m8 = __ballot(in8), m4 = __ballot(in4);
      if (m8) {
        uint32_t at = 0;
        if (lane == 0) at = atomicAdd(&ncand[0], (uint32_t)__builtin_popcountll(m8));
        at = __shfl(at, 0, 64) + __builtin_amdgcn_mbcnt_hi((uint32_t)(m8 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m8, 0u));
        if (in8 && at < kCap) cand[0][at] = v;
      }
      if (m4) {
        uint32_t at = 0;
        if (lane == 0) at = atomicAdd(&ncand[1], (uint32_t)__builtin_popcountll(m4));
        at = __shfl(at, 0, 64) + __builtin_amdgcn_mbcnt_hi((uint32_t)(m4 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m4, 0u));
        if (in4 && at < kCap) cand[1][at] = v;
      }
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      always4 += __shfl_xor(always4, d, 64);
      if constexpr (WIDE) always8 += __shfl_xor(always8, d, 64);
    }
    if (lane == 0) {
      red[0][0][wave] = always4;
      if constexpr (WIDE) red[0][1][wave] = always8;
    }
    __syncthreads();
    const uint32_t n8 = ncand[0], n4 = ncand[1];
    if constexpr (!WIDE) base8 = hist[b_fit];  // patterns at or above hi: exact, hi is a bin boundary
#pragma unroll
    for (int w = 0; w < kAllocWaves; ++w) {
      base4 += red[0][0][w];
      if constexpr (WIDE) base8 += red[0][1][w];
    }
    narrowed = n8 <= kCap && n4 <= kCap;  // otherwise (masses of equal values) count everything again
    __syncthreads();                      // red is reused below
    if (narrowed) {
      // (4) bisection over the candidates
      while (hi - lo > 1) {
        const uint32_t mid = lo + (hi - lo) / 2;
        const int32_t m8 = (int32_t)mid, m4 = (int32_t)p4_of(mid);
        uint32_t a4 = 0, a8 = 0;
        for (uint32_t i = tid; i < n8; i += kAllocThreads) a8 += cand[0][i] >= m8 ? 1u : 0u;
        for (uint32_t i = tid; i < n4; i += kAllocThreads) a4 += cand[1][i] >= m4 ? 1u : 0u;
        uint32_t both = a4 | (a8 << 16);  // at most kCap / 1024 each per lane
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) both += __shfl_xor(both, d, 64);
        if (lane == 0) red[turn][0][wave] = both;
        __syncthreads();
        uint32_t s4 = base4, s8 = base8;
#pragma unroll
        for (int w = 0; w < kAllocWaves; ++w) {
          const uint32_t t = red[turn][0][w];
          s4 += t & 0xFFFFu;
          s8 += t >> 16;
        }
        turn ^= 1u;
        const uint64_t cost = 2ull * J + 2ull * s4 + 4ull * s8;
        if (cost <= max_code_bits) hi = mid; else lo = mid;
      }
    }
  }
  }
  if (!narrowed) {
    while (hi - lo > 1) {
      const uint32_t mid = lo + (hi - lo) / 2;
      uint32_t s4, s8, s16;
      block_counts(mid, s4, s8, s16);
      const uint64_t cost = 2ull * J + 2ull * s4 + 4ull * s8 + 8ull * s16;
      if (cost <= max_code_bits) hi = mid; else lo = mid;
    }
  }
  uint32_t s4, s8, s16;
  block_counts(hi, s4, s8, s16);
  const int32_t p8 = (int32_t)hi, p4 = p4_from(hi), p16 = p16_from(hi, allow16);
  const uint32_t n_class[4] = {J - s4, s4 - s8, s8 - s16, s16};
  if constexpr (WIDE) {
    if (tid == 0) {
      uint32_t *cnt = counts_all + 5ull * blockIdx.x;
      gst<uint32_t>(cnt, n_class[0]);
      gst<uint32_t>(cnt + 1, n_class[1]);
      gst<uint32_t>(cnt + 2, n_class[2]);
      gst<uint32_t>(cnt + 3, n_class[3]);
      gst<uint32_t>(cnt + 4, hi);
    }
    return;
  }
  // first position of each class in the reordered bucket, advanced chunk by chunk
  uint32_t next[4] = {0, n_class[0], n_class[0] + n_class[1], n_class[0] + n_class[1] + n_class[2]};

  // Positions of the stable reorder, 64 rows of 1024 super-groups at a time: the rank of a
  // super-group inside its class is (members in earlier rows and waves) + (members in lower lanes).
  for (uint32_t r0 = 0; r0 < rows; r0 += kRegs) {
    const uint32_t nr = min((uint32_t)kRegs, rows - r0);
    auto slot = [&](uint32_t k) -> int32_t {  // buckets too large for registers: read again
      const uint32_t j = (r0 + k) * kAllocThreads + tid;
      return j < J ? pattern_of(gld<float>(F + j)) : -1;
    };
    // pass 1: class counts of every (row, wave)
    if constexpr (IN_REGS) {
#pragma unroll
      for (int k = 0; k < kRegs; ++k) {
        if ((uint32_t)k < nr) {
          const uint32_t c = class_of(fr[k], p4, p8, p16);
          const uint64_t b0 = __ballot(c == 0), b1 = __ballot(c == 1), b2 = __ballot(c == 2), b3 = __ballot(c == 3);
          if (lane == 0) {
            tot[k * kAllocWaves + wave][0] = (uint32_t)__builtin_popcountll(b0);
            tot[k * kAllocWaves + wave][1] = (uint32_t)__builtin_popcountll(b1);
            tot[k * kAllocWaves + wave][2] = (uint32_t)__builtin_popcountll(b2);
            tot[k * kAllocWaves + wave][3] = (uint32_t)__builtin_popcountll(b3);
          }
        }
      }
    } else {
      for (uint32_t k = 0; k < nr; ++k) {
        const uint32_t c = class_of(slot(k), p4, p8, p16);
        const uint64_t b0 = __ballot(c == 0), b1 = __ballot(c == 1), b2 = __ballot(c == 2), b3 = __ballot(c == 3);
        if (lane == 0) {
          tot[k * kAllocWaves + wave][0] = (uint32_t)__builtin_popcountll(b0);
          tot[k * kAllocWaves + wave][1] = (uint32_t)__builtin_popcountll(b1);
          tot[k * kAllocWaves + wave][2] = (uint32_t)__builtin_popcountll(b2);
          tot[k * kAllocWaves + wave][3] = (uint32_t)__builtin_popcountll(b3);
        }
      }
    }
    __syncthreads();
    // pass 2: exclusive scan of the counts in (row, wave) order; thread e owns entry e
    uint32_t x[4], inc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      x[c] = tid < nr * kAllocWaves ? tot[tid][c] : 0u;
      inc[c] = x[c];
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = __shfl_up(inc[c], d, 64);
        if (lane >= (uint32_t)d) inc[c] += up;
      }
      if (lane == 63) wsum[wave][c] = inc[c];
    }
    __syncthreads();
    uint32_t chunk_total[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      uint32_t before = 0, all = 0;
#pragma unroll
      for (int w = 0; w < kAllocWaves; ++w) {
        const uint32_t t = wsum[w][c];
        before += (uint32_t)w < wave ? t : 0u;
        all += t;
      }
      chunk_total[c] = all;
      if (tid < nr * kAllocWaves) tot[tid][c] = next[c] + before + inc[c] - x[c];
    }
    __syncthreads();
    // pass 3: widths and positions, coalesced
    auto emit = [&](uint32_t k, int32_t v) {
      const uint32_t j = (r0 + k) * kAllocThreads + tid;
      const uint32_t c = class_of(v, p4, p8, p16);
      const uint64_t b0 = __ballot(c == 0), b1 = __ballot(c == 1), b2 = __ballot(c == 2), b3 = __ballot(c == 3);
      const uint64_t mine = c == 0 ? b0 : (c == 1 ? b1 : (c == 2 ? b2 : b3));
      const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mine >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mine, 0u));
      if (c < 4) {
        gst<uint8_t>(widths + j, (uint8_t)(2u << c));
        gst<uint32_t>(pos + j, tot[k * kAllocWaves + wave][c] + rank);
      }
    };
    if constexpr (IN_REGS) {
#pragma unroll
      for (int k = 0; k < kRegs; ++k)
        if ((uint32_t)k < nr) emit(k, fr[k]);
    } else {
      for (uint32_t k = 0; k < nr; ++k) emit(k, slot(k));
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) next[c] += chunk_total[c];
    __syncthreads();  // tot and wsum are reused by the next chunk
  }
  if (tid == 0) {
    uint32_t *cnt = counts_all + 5ull * blockIdx.x;
    gst<uint32_t>(cnt, n_class[0]);
    gst<uint32_t>(cnt + 1, n_class[1]);
    gst<uint32_t>(cnt + 2, n_class[2]);
    gst<uint32_t>(cnt + 3, n_class[3]);
    gst<uint32_t>(cnt + 4, hi);
  }
}

// ---------------------------------------------------------------------------------------
// Reorder and restore move whole super-groups in 16-byte pieces: piece c of the source
// belongs to super-group c / pps (pps = pieces per SG) and lands at the same offset inside
// the destination super-group.  Each thread moves kUnroll pieces per round, 1 KB apart, so a
// wave has 4 KB in flight.
constexpr int kUnroll = 4;

template <uint32_t PPS>  // 16-byte pieces per super-group: 64 (fp32) or 32 (bf16)
__global__ void __launch_bounds__(kThreads) k_reorder(const void *x_all, const uint32_t *pos_all, uint32_t J, void *out_all) {
  const uint64_t bucket_first = (uint64_t)blockIdx.y * J;  // blockIdx.y = bucket
  const uint8_t *x = static_cast<const uint8_t *>(x_all) + bucket_first * PPS * 16;
  uint8_t *out = static_cast<uint8_t *>(out_all) + bucket_first * PPS * 16;
  const uint32_t *pos = pos_all + bucket_first;
  const uint32_t n_pieces = J * PPS;
  const uint32_t stride = gridDim.x * kThreads * kUnroll;
  for (uint32_t base = blockIdx.x * kThreads * kUnroll + threadIdx.x; base < n_pieces; base += stride) {
    u32x4 d[kUnroll];
    uint32_t dst[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const uint32_t c = base + i * kThreads;
      if (c < n_pieces) {
        d[i] = gld<u32x4>(x + (uint64_t)c * 16);
        dst[i] = gld<uint32_t>(pos + c / PPS) * PPS + c % PPS;
      }
    }
#pragma unroll
    for (int i = 0; i < kUnroll; ++i)
      if (base + i * kThreads < n_pieces) gst<u32x4>(out + (uint64_t)dst[i] * 16, d[i]);
  }
}

// The means the main stage subtracts, in reordered order; zero for the 16-bit super-groups (the
// last counts[5b + 3] places of bucket b); and the inverse of the positions.  One thread per super-group.
__global__ void __launch_bounds__(kThreads) k_reorder_mean(const float *mu_all, const uint32_t *pos_all, const uint32_t *counts,
                                                           uint32_t J, float *mu_main, uint32_t *origin) {
  const uint64_t bucket_first = (uint64_t)blockIdx.y * J;
  const uint32_t n16 = counts ? gld<uint32_t>(counts + 5ull * blockIdx.y + 3) : 0u;
  for (uint32_t j = blockIdx.x * kThreads + threadIdx.x; j < J; j += gridDim.x * kThreads) {
    const uint32_t p = gld<uint32_t>(pos_all + bucket_first + j);
    if (mu_main) {
      const float m = gld<float>(mu_all + bucket_first + j);
      gst<float>(mu_main + bucket_first + p, (p < J - n16) ? m : 0.0f);
    }
    if (origin) gst<uint32_t>(origin + bucket_first + p, j);
  }
}

__global__ void __launch_bounds__(kThreads) k_restore(const float *sum_all, const uint32_t *pos_all, const float *mu_all,
                                                      float n, uint32_t J, float *out_all) {
  constexpr uint32_t pps = kSG * 4 / 16;
  const uint64_t bucket_first = (uint64_t)blockIdx.y * J;
  const uint8_t *sum = reinterpret_cast<const uint8_t *>(sum_all) + bucket_first * pps * 16;
  uint8_t *out = reinterpret_cast<uint8_t *>(out_all) + bucket_first * pps * 16;
  const uint32_t *pos = pos_all + bucket_first;
  const float *mu = mu_all ? mu_all + bucket_first : nullptr;  // in reordered order
  const uint32_t n_pieces = J * pps;
  const uint32_t stride = gridDim.x * kThreads * kUnroll;
  for (uint32_t base = blockIdx.x * kThreads * kUnroll + threadIdx.x; base < n_pieces; base += stride) {
    f32x4 d[kUnroll];
    float back[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const uint32_t c = base + i * kThreads;
      if (c < n_pieces) {
        const uint32_t p = gld<uint32_t>(pos + c / pps);
        d[i] = gld<f32x4>(sum + ((uint64_t)p * pps + c % pps) * 16);
        back[i] = mu ? n * gld<float>(mu + p) : 0.0f;
      }
    }
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const uint32_t c = base + i * kThreads;
      if (c < n_pieces) {
        f32x4 o = d[i];
        if (mu) { o.x = d[i].x + back[i]; o.y = d[i].y + back[i]; o.z = d[i].z + back[i]; o.w = d[i].w + back[i]; }
        gst<f32x4>(out + (uint64_t)c * 16, o);
      }
    }
  }
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// blocks per grid row: enough for the units of one row, at most the GPU's resident share
uint32_t stream_blocks(uint64_t units_per_block_round, uint64_t units, uint32_t rows = 1) {
  int dev = 0, n_cu = 256;
  if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  const uint64_t need = (units + units_per_block_round - 1) / units_per_block_round;
  const uint64_t cap = ((uint64_t)n_cu * 8 + rows - 1) / rows;  // 8 blocks of 256 threads per CU in all
  return (uint32_t)(need < 1 ? 1 : (need < cap ? need : cap));
}

dq_status launched() { return dq::hip_status(hipGetLastError()); }

}  // namespace

extern "C" {

dq_status dq_sg_stats(const void *x, dq_dtype dtype, uint64_t n_sg, float *mu_out, float *F_out, void *hip_stream) {
  if (n_sg == 0) return DQ_OK;
  if (!x || !mu_out || !F_out || (dtype != DQ_F32 && dtype != DQ_BF16)) return DQ_EINVAL;
  if (!aligned(x, 16) || !aligned(mu_out, 4) || !aligned(F_out, 4)) return DQ_EALIGN;
  const uint32_t blocks = stream_blocks(4 * (kThreads / 64), n_sg);
  hipStream_t s = (hipStream_t)hip_stream;
  if (dtype == DQ_F32) hipLaunchKernelGGL(k_stats<float>, dim3(blocks), dim3(kThreads), 0, s, x, n_sg, mu_out, F_out);
  else hipLaunchKernelGGL(k_stats<uint16_t>, dim3(blocks), dim3(kThreads), 0, s, x, n_sg, mu_out, F_out);
  return launched();
}

dq_status dq_stats_combine(const float *mu_all, const float *F_all, uint32_t n_workers, uint64_t n_sg, float *mu,
                           float *F, void *hip_stream) {
  if (n_sg == 0) return DQ_OK;
  if (!mu_all || !F_all || !mu || !F || n_workers == 0) return DQ_EINVAL;
  if (!aligned(mu_all, 4) || !aligned(F_all, 4) || !aligned(mu, 4) || !aligned(F, 4)) return DQ_EALIGN;
  if ((n_sg + kThreads - 1) / kThreads > 0x7FFFFFFFull) return DQ_EUNSUPPORTED;
  hipLaunchKernelGGL(k_combine, dim3((uint32_t)((n_sg + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                     (hipStream_t)hip_stream, mu_all, F_all, n_workers, n_sg, mu, F);
  return launched();
}

dq_status dq_allocate(const float *F, uint32_t n_sg_per_bucket, uint32_t n_buckets, uint64_t max_code_bits,
                      uint32_t max_width, uint8_t *widths, uint32_t *pos, uint32_t *counts, void *hip_stream) {
  if (n_sg_per_bucket == 0 || n_buckets == 0) return DQ_OK;
  if (!F || !widths || !pos || !counts || (max_width != 8 && max_width != 16)) return DQ_EINVAL;
  if (max_code_bits < 2ull * n_sg_per_bucket) return DQ_EINVAL;  // fewer than 2 code bits per coordinate
  if (!aligned(F, 4) || !aligned(pos, 4) || !aligned(counts, 4)) return DQ_EALIGN;
  hipStream_t s = (hipStream_t)hip_stream;
  if (n_sg_per_bucket <= (uint32_t)kRegs * kAllocThreads)
    hipLaunchKernelGGL(k_allocate<true>, dim3(n_buckets), dim3(kAllocThreads), 0, s, F, n_sg_per_bucket, max_code_bits,
                       max_width == 16, widths, pos, counts);
  else
    hipLaunchKernelGGL(k_allocate<false>, dim3(n_buckets), dim3(kAllocThreads), 0, s, F, n_sg_per_bucket, max_code_bits,
                       max_width == 16, widths, pos, counts);
  return launched();
}

// Blocks per bucket of the two histogram levels: one per 4096 super-groups, at most 8 (the next
// launch adds up that many records per block).
static uint32_t wide_blocks(uint32_t n_sg_per_bucket) {
  const uint32_t g = (n_sg_per_bucket + 4095u) / 4096u;
  return g < 1 ? 1 : (g > kMaxLevelBlocks ? kMaxLevelBlocks : g);
}
static bool wide_applies(uint32_t n_sg_per_bucket, uint32_t n_buckets, uint32_t max_width) {
  return max_width == 8 && n_sg_per_bucket <= (uint32_t)kRegs * kAllocThreads && n_buckets <= 65535u;
}

size_t dq_allocate_wide_workspace_bytes(uint32_t n_sg_per_bucket, uint32_t n_buckets) {
  const size_t words = 2 * (size_t)wide_blocks(n_sg_per_bucket) * kPartWords + 4;  // two levels' records, the bracket
  return (size_t)n_buckets * words * sizeof(uint32_t);
}

dq_status dq_allocate_wide(const float *F, uint32_t n_sg_per_bucket, uint32_t n_buckets, uint64_t max_code_bits,
                           uint32_t max_width, uint8_t *widths, uint32_t *pos, uint32_t *counts, void *workspace,
                           size_t workspace_bytes, void *hip_stream) {
  if (n_sg_per_bucket == 0 || n_buckets == 0) return DQ_OK;
  if (!wide_applies(n_sg_per_bucket, n_buckets, max_width))
    return dq_allocate(F, n_sg_per_bucket, n_buckets, max_code_bits, max_width, widths, pos, counts, hip_stream);
  if (!F || !widths || !pos || !counts || !workspace) return DQ_EINVAL;
  if (max_code_bits < 2ull * n_sg_per_bucket) return DQ_EINVAL;
  if (workspace_bytes < dq_allocate_wide_workspace_bytes(n_sg_per_bucket, n_buckets)) return DQ_EINVAL;
  if (!aligned(F, 4) || !aligned(pos, 4) || !aligned(counts, 4) || !aligned(workspace, 16)) return DQ_EALIGN;
  hipStream_t s = (hipStream_t)hip_stream;
  const uint32_t G = wide_blocks(n_sg_per_bucket);
  uint32_t *part1 = static_cast<uint32_t *>(workspace);
  uint32_t *part2 = part1 + (size_t)n_buckets * G * kPartWords;
  uint32_t *ctl = part2 + (size_t)n_buckets * G * kPartWords;
  hipLaunchKernelGGL(k_alloc_level<true>, dim3(G, n_buckets), dim3(kLevelThreads), 0, s, F, n_sg_per_bucket, max_code_bits,
                     (const uint32_t *)nullptr, part1, ctl);
  hipLaunchKernelGGL(k_alloc_level<false>, dim3(G, n_buckets), dim3(kLevelThreads), 0, s, F, n_sg_per_bucket, max_code_bits,
                     (const uint32_t *)part1, part2, ctl);
  hipLaunchKernelGGL((k_allocate<true, true>), dim3(n_buckets), dim3(kAllocThreads), 0, s, F, n_sg_per_bucket, max_code_bits,
                     false, widths, pos, counts, (const uint32_t *)part2, G, (const uint32_t *)ctl);
  hipLaunchKernelGGL(k_alloc_positions, dim3((n_sg_per_bucket + kAllocThreads - 1) / kAllocThreads, n_buckets),
                     dim3(kAllocThreads), 0, s, F, n_sg_per_bucket, (const uint32_t *)counts, widths, pos);
  return launched();
}

dq_status dq_reorder(const void *x, dq_dtype dtype, const uint32_t *pos, uint32_t n_sg_per_bucket, uint32_t n_buckets,
                     void *out, void *hip_stream) {
  if (n_sg_per_bucket == 0 || n_buckets == 0) return DQ_OK;
  if (!x || !pos || !out || x == out || (dtype != DQ_F32 && dtype != DQ_BF16)) return DQ_EINVAL;
  if (n_sg_per_bucket > (1u << 24) || n_buckets > 65535u) return DQ_EUNSUPPORTED;
  if (!aligned(x, 16) || !aligned(out, 16) || !aligned(pos, 4)) return DQ_EALIGN;
  const uint64_t pieces = (uint64_t)n_sg_per_bucket * (dtype == DQ_F32 ? 64 : 32);
  const uint32_t blocks = stream_blocks((uint64_t)kThreads * kUnroll, pieces, n_buckets);
  hipStream_t s = (hipStream_t)hip_stream;
  if (dtype == DQ_F32)
    hipLaunchKernelGGL(k_reorder<64>, dim3(blocks, n_buckets), dim3(kThreads), 0, s, x, pos, n_sg_per_bucket, out);
  else
    hipLaunchKernelGGL(k_reorder<32>, dim3(blocks, n_buckets), dim3(kThreads), 0, s, x, pos, n_sg_per_bucket, out);
  return launched();
}

dq_status dq_reorder_mean(const float *mu_or_null, const uint32_t *pos, const uint32_t *counts_or_null,
                          uint32_t n_sg_per_bucket, uint32_t n_buckets, float *mu_main_or_null, uint32_t *origin_or_null,
                          void *hip_stream) {
  if (n_sg_per_bucket == 0 || n_buckets == 0) return DQ_OK;
  if (!pos || (!mu_main_or_null && !origin_or_null) || (mu_main_or_null && (!mu_or_null || mu_or_null == mu_main_or_null)) ||
      origin_or_null == pos)
    return DQ_EINVAL;
  if (n_sg_per_bucket > (1u << 24) || n_buckets > 65535u) return DQ_EUNSUPPORTED;
  if (!aligned(mu_or_null, 4) || !aligned(pos, 4) || !aligned(counts_or_null, 4) || !aligned(mu_main_or_null, 4) ||
      !aligned(origin_or_null, 4))
    return DQ_EALIGN;
  const uint32_t blocks = stream_blocks(kThreads, n_sg_per_bucket, n_buckets);
  hipLaunchKernelGGL(k_reorder_mean, dim3(blocks, n_buckets), dim3(kThreads), 0, (hipStream_t)hip_stream, mu_or_null, pos,
                     counts_or_null, n_sg_per_bucket, mu_main_or_null, origin_or_null);
  return launched();
}

dq_status dq_restore(const float *sum, const uint32_t *pos, const float *mu_main_or_null, uint32_t n_workers,
                     uint32_t n_sg_per_bucket, uint32_t n_buckets, float *out, void *hip_stream) {
  if (n_sg_per_bucket == 0 || n_buckets == 0) return DQ_OK;
  if (!sum || !pos || !out || sum == out || n_workers == 0) return DQ_EINVAL;
  if (n_sg_per_bucket > (1u << 24) || n_buckets > 65535u) return DQ_EUNSUPPORTED;
  if (!aligned(sum, 16) || !aligned(out, 16) || !aligned(pos, 4) || !aligned(mu_main_or_null, 4)) return DQ_EALIGN;
  const uint32_t blocks = stream_blocks((uint64_t)kThreads * kUnroll, (uint64_t)n_sg_per_bucket * 64, n_buckets);
  hipLaunchKernelGGL(k_restore, dim3(blocks, n_buckets), dim3(kThreads), 0, (hipStream_t)hip_stream, sum, pos,
                     mu_main_or_null, (float)n_workers, n_sg_per_bucket, out);
  return launched();
}

}  // extern "C"
