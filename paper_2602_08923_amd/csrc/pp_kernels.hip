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

// Widths and positions once the threshold is known (counts[5b..5b+4] as the search left them):
// grid (ceil(J / 1024), buckets).  A block first counts the members of each class among the
// super-groups before its own 1024 (at most 64 rows for the sizes this path takes), then ranks
// its own: position = first place of the class + members before the block + members in earlier
// waves + members in lower lanes.
__global__ void __launch_bounds__(kAllocThreads) k_alloc_positions(const float *F_all, uint32_t J, bool allow16,
                                                                   const uint32_t *counts_all, uint8_t *widths_all,
                                                                   uint32_t *pos_all) {
  __shared__ uint32_t before[kAllocWaves][4], mine_w[kAllocWaves][4];
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint64_t first = (uint64_t)blockIdx.y * J;
  const float *F = F_all + first;
  const uint32_t *cnt = counts_all + 5ull * blockIdx.y;
  const uint32_t pattern = gld<uint32_t>(cnt + 4);
  const int32_t p8 = (int32_t)pattern, p4 = p4_from(pattern), p16 = p16_from(pattern, allow16);
  const uint32_t n0 = gld<uint32_t>(cnt), n1 = gld<uint32_t>(cnt + 1), n2 = gld<uint32_t>(cnt + 2);
  const uint32_t start[4] = {0u, n0, n0 + n1, n0 + n1 + n2};
  uint32_t c[4] = {0u, 0u, 0u, 0u};
  constexpr uint32_t kAhead = 32;  // rows of 1024 before this block, that many loads in flight
  for (uint32_t r0 = 0; r0 < blockIdx.x; r0 += kAhead) {
    float f[kAhead];
#pragma unroll
    for (uint32_t r = 0; r < kAhead; ++r) f[r] = gld<float>(F + min(r0 + r, blockIdx.x - 1) * kAllocThreads + tid);
#pragma unroll
    for (uint32_t r = 0; r < kAhead; ++r) {
      const uint32_t k = r0 + r < blockIdx.x ? class_of(pattern_of(f[r]), p4, p8, p16) : 4u;
#pragma unroll
      for (uint32_t i = 0; i < 4; ++i) c[i] += k == i ? 1u : 0u;
    }
  }
  const uint32_t j = blockIdx.x * kAllocThreads + tid;
  const uint32_t k = j < J ? class_of(pattern_of(gld<float>(F + j)), p4, p8, p16) : 4u;
  const uint64_t b[4] = {__ballot(k == 0), __ballot(k == 1), __ballot(k == 2), __ballot(k == 3)};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) c[i] += __shfl_xor(c[i], d, 64);
  }
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      before[wave][i] = c[i];
      mine_w[wave][i] = (uint32_t)__builtin_popcountll(b[i]);
    }
  }
  __syncthreads();
  if (k < 4) {
    uint32_t at = start[k];
#pragma unroll
    for (int w = 0; w < kAllocWaves; ++w) at += before[w][k] + ((uint32_t)w < wave ? mine_w[w][k] : 0u);
    const uint64_t mine = k == 0 ? b[0] : (k == 1 ? b[1] : (k == 2 ? b[2] : b[3]));
    at += __builtin_amdgcn_mbcnt_hi((uint32_t)(mine >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mine, 0u));
    gst<uint8_t>(widths_all + first + j, (uint8_t)(2u << k));
    gst<uint32_t>(pos_all + first + j, at);
  }
}

// IN_REGS (buckets of at most 65,536 super-groups): the kernel ends once counts[5b..5b+4] are
// written, widths and positions are another launch (k_alloc_positions, spread over the GPU: ranking
// 64 rows in this one block took longer than the whole search and spilled registers); larger
// buckets do them here, 64 rows of 1024 at a time, reading the norms again.
template <bool IN_REGS>
__global__ void __launch_bounds__(kAllocThreads) k_allocate(const float *F_all, uint32_t J, uint64_t max_code_bits,
                                                            bool allow16, uint8_t *widths_all, uint32_t *pos_all,
                                                            uint32_t *counts_all) {
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
    uint32_t b_no = 0, b_fit = kBins - 8;  // 2040: +infinity, everything at 2 bits
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
    // (3) Only patterns strictly inside (lo, hi) can change c8 while the threshold moves in
    //     (lo, hi], and only patterns in [p4(lo), p4(hi)) can change c4: collect them in LDS.
    const int32_t lo8 = (int32_t)lo, hi8 = (int32_t)hi, lo4 = (int32_t)p4_of(lo), hi4 = (int32_t)p4_of(hi);
    if (tid < 2) ncand[tid] = 0;
    __syncthreads();
    uint32_t always4 = 0;
#pragma unroll
    for (int k = 0; k < kRegs; ++k) {
      const int32_t v = fr[k];
      const bool in8 = v > lo8 && v < hi8, in4 = v >= lo4 && v < hi4;
      always4 += v >= hi4 ? 1u : 0u;
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
    for (int d = 1; d < 64; d <<= 1) always4 += __shfl_xor(always4, d, 64);
    if (lane == 0) red[0][0][wave] = always4;
    __syncthreads();
    const uint32_t n8 = ncand[0], n4 = ncand[1];
    base8 = hist[b_fit];  // patterns at or above hi: exact, hi is a bin boundary
#pragma unroll
    for (int w = 0; w < kAllocWaves; ++w) base4 += red[0][0][w];
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
  if constexpr (IN_REGS) {
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

  // Positions of the stable reorder (buckets too large for registers), 64 rows of 1024 super-groups
  // at a time, the norms read again: the rank of a super-group inside its class is (members in
  // earlier rows and waves) + (members in lower lanes).
  for (uint32_t r0 = 0; r0 < rows; r0 += kRegs) {
    const uint32_t nr = min((uint32_t)kRegs, rows - r0);
    auto slot = [&](uint32_t k) -> int32_t {
      const uint32_t j = (r0 + k) * kAllocThreads + tid;
      return j < J ? pattern_of(gld<float>(F + j)) : -1;
    };
    // pass 1: class counts of every (row, wave)
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
    for (uint32_t k = 0; k < nr; ++k) emit(k, slot(k));
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

// k_alloc_positions over all buckets, 65,535 (the grid's second dimension) per launch
static void launch_positions(const float *F, uint32_t J, uint32_t n_buckets, bool allow16, const uint32_t *counts,
                             uint8_t *widths, uint32_t *pos, hipStream_t s) {
  for (uint32_t b0 = 0; b0 < n_buckets; b0 += 65535u) {
    const uint32_t nb = n_buckets - b0 < 65535u ? n_buckets - b0 : 65535u;
    const uint64_t off = (uint64_t)b0 * J;
    hipLaunchKernelGGL(k_alloc_positions, dim3((J + kAllocThreads - 1) / kAllocThreads, nb), dim3(kAllocThreads), 0, s,
                       F + off, J, allow16, counts + 5ull * b0, widths + off, pos + off);
  }
}

dq_status dq_allocate(const float *F, uint32_t n_sg_per_bucket, uint32_t n_buckets, uint64_t max_code_bits,
                      uint32_t max_width, uint8_t *widths, uint32_t *pos, uint32_t *counts, void *hip_stream) {
  if (n_sg_per_bucket == 0 || n_buckets == 0) return DQ_OK;
  if (!F || !widths || !pos || !counts || (max_width != 8 && max_width != 16)) return DQ_EINVAL;
  if (max_code_bits < 2ull * n_sg_per_bucket) return DQ_EINVAL;  // fewer than 2 code bits per coordinate
  if (!aligned(F, 4) || !aligned(pos, 4) || !aligned(counts, 4)) return DQ_EALIGN;
  hipStream_t s = (hipStream_t)hip_stream;
  if (n_sg_per_bucket <= (uint32_t)kRegs * kAllocThreads) {
    // the search in one block per bucket, the norms in registers; widths and positions on a grid
    hipLaunchKernelGGL(k_allocate<true>, dim3(n_buckets), dim3(kAllocThreads), 0, s, F, n_sg_per_bucket, max_code_bits,
                       max_width == 16, widths, pos, counts);
    launch_positions(F, n_sg_per_bucket, n_buckets, max_width == 16, counts, widths, pos, s);
  } else
    hipLaunchKernelGGL(k_allocate<false>, dim3(n_buckets), dim3(kAllocThreads), 0, s, F, n_sg_per_bucket, max_code_bits,
                       max_width == 16, widths, pos, counts);
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
