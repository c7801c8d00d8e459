// Steps before and after the main all-reduce stage, for gfx950: per-super-group statistics
// (Section 3.1), their combination over workers with the bf16 exchange format (Sections 3.1,
// 3.5), the three-width bit allocation with tied thresholds (Section 3.2, Appendix A), the
// mean-subtracting reorder into increasing width order (Sections 3.1, 3.5) and the final
// restore (Section 3.4, last paragraph).  All of them stream each entry once; the allocation
// works on 4 bytes per super-group.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dq.h"

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
// Allocation: one block of 1024 threads per bucket.  Thread t owns the run of `per`
// consecutive super-groups starting at t*per (in registers when per <= kRegs), so that the
// positions of the stable reorder follow from one block-wide exclusive scan.
constexpr int kAllocThreads = 1024;
constexpr int kRegs = 64;

__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t *lds) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) v += __shfl_xor(v, d, 64);
  const uint32_t wave = threadIdx.x >> 6;
  __syncthreads();  // the previous round's readers are done
  if ((threadIdx.x & 63u) == 0) lds[wave] = v;
  __syncthreads();
  uint32_t tot = 0;
#pragma unroll
  for (int w = 0; w < kAllocThreads / 64; ++w) tot += lds[w];
  return tot;
}

// widths follow Section 3.2's tied thresholds: T_{2,4} = 17/512 * T_{4,8}
__device__ __forceinline__ uint32_t width_of(float F, float theta, float t24) {
  return F >= theta ? 8u : (F >= t24 ? 4u : 2u);
}

template <bool IN_REGS>
__global__ void __launch_bounds__(kAllocThreads) k_allocate(const float *F_all, uint32_t J, uint64_t max_code_bits,
                                                            uint8_t *widths_all, uint32_t *pos_all, uint32_t *counts_all) {
  __shared__ uint32_t red[kAllocThreads / 64];
  __shared__ uint32_t scan[3][kAllocThreads / 64];
  const float *F = F_all + (uint64_t)blockIdx.x * J;
  uint8_t *widths = widths_all + (uint64_t)blockIdx.x * J;
  uint32_t *pos = pos_all + (uint64_t)blockIdx.x * J;
  const uint32_t per = (J + kAllocThreads - 1) / kAllocThreads;
  const uint32_t j0 = min(threadIdx.x * per, J), j1 = min(j0 + per, J);
  float fr[IN_REGS ? kRegs : 1];
  if constexpr (IN_REGS) {
#pragma unroll
    for (int k = 0; k < kRegs; ++k) fr[k] = (j0 + k < j1) ? gld<float>(F + j0 + k) : -1.0f;  // -1: below any threshold
  }
  auto count = [&](float theta, uint32_t &c4, uint32_t &c8) {
    const float t24 = theta * (17.0f / 512.0f);
    c4 = 0; c8 = 0;
    if constexpr (IN_REGS) {
#pragma unroll
      for (int k = 0; k < kRegs; ++k) {
        c4 += fr[k] >= t24 ? 1u : 0u;
        c8 += fr[k] >= theta ? 1u : 0u;
      }
    } else {
      for (uint32_t j = j0; j < j1; ++j) {
        const float f = gld<float>(F + j);
        c4 += f >= t24 ? 1u : 0u;
        c8 += f >= theta ? 1u : 0u;
      }
    }
  };
  // smallest fp32 pattern in [1, +inf] whose allocation fits; the host has checked 2J <= budget.
  // An SG at or above T_{4,8} is also at or above T_{2,4}: cost = 2J + 2*c4 + 4*c8.
  uint32_t lo = 0, hi = 0x7F800000u;
  while (hi - lo > 1) {
    const uint32_t mid = lo + (hi - lo) / 2;
    uint32_t c4, c8;
    count(u2f(mid), c4, c8);
    const uint32_t s4 = block_sum(c4, red);
    const uint32_t s8 = block_sum(c8, red);
    const uint64_t cost = 2ull * J + 2ull * s4 + 4ull * s8;
    if (cost <= max_code_bits) hi = mid; else lo = mid;
  }
  const float theta = u2f(hi), t24 = theta * (17.0f / 512.0f);
  // class counts of the thread's run, then exclusive scans over the block
  uint32_t n[3] = {0, 0, 0};
  if constexpr (IN_REGS) {
#pragma unroll
    for (int k = 0; k < kRegs; ++k)
      if (j0 + k < j1) {
        const uint32_t w = width_of(fr[k], theta, t24);
        n[w == 2 ? 0 : w == 4 ? 1 : 2] += 1;
      }
  } else {
    for (uint32_t j = j0; j < j1; ++j) {
      const uint32_t w = width_of(gld<float>(F + j), theta, t24);
      n[w == 2 ? 0 : w == 4 ? 1 : 2] += 1;
    }
  }
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  uint32_t excl[3], total[3];
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    uint32_t inc = n[c];
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t up = __shfl_up(inc, d, 64);
      if (lane >= (uint32_t)d) inc += up;
    }
    if (lane == 63) scan[c][wave] = inc;
    excl[c] = inc - n[c];
  }
  __syncthreads();
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kAllocThreads / 64; ++w) {
      const uint32_t s = scan[c][w];
      before += (uint32_t)w < wave ? s : 0u;
      all += s;
    }
    excl[c] += before;
    total[c] = all;
  }
  uint32_t next[3] = {excl[0], total[0] + excl[1], total[0] + total[1] + excl[2]};
  if constexpr (IN_REGS) {
#pragma unroll
    for (int k = 0; k < kRegs; ++k)
      if (j0 + k < j1) {
        const uint32_t w = width_of(fr[k], theta, t24);
        const int c = w == 2 ? 0 : w == 4 ? 1 : 2;
        gst<uint8_t>(widths + j0 + k, (uint8_t)w);
        gst<uint32_t>(pos + j0 + k, next[c]);
        next[c] += 1;
      }
  } else {
    for (uint32_t j = j0; j < j1; ++j) {
      const uint32_t w = width_of(gld<float>(F + j), theta, t24);
      const int c = w == 2 ? 0 : w == 4 ? 1 : 2;
      gst<uint8_t>(widths + j, (uint8_t)w);
      gst<uint32_t>(pos + j, next[c]);
      next[c] += 1;
    }
  }
  if (threadIdx.x == 0) {
    uint32_t *cnt = counts_all + 4ull * blockIdx.x;
    gst<uint32_t>(cnt, total[0]);
    gst<uint32_t>(cnt + 1, total[1]);
    gst<uint32_t>(cnt + 2, total[2]);
    gst<uint32_t>(cnt + 3, hi);
  }
}

// ---------------------------------------------------------------------------------------
// Reorder and restore move whole super-groups in 16-byte pieces: piece c of the source
// belongs to super-group c / pps (pps = pieces per SG) and lands at the same offset inside
// the destination super-group.  Each thread moves kUnroll pieces per round, 1 KB apart, so a
// wave has 4 KB in flight.
constexpr int kUnroll = 4;

template <typename LT>
__global__ void __launch_bounds__(kThreads) k_reorder(const void *x_all, const uint32_t *pos_all, const float *mu_all,
                                                      uint32_t J, void *out_all) {
  constexpr uint32_t pps = kSG * sizeof(LT) / 16;
  const uint64_t bucket_first = (uint64_t)blockIdx.y * J;  // blockIdx.y = bucket
  const uint8_t *x = static_cast<const uint8_t *>(x_all) + bucket_first * pps * 16;
  uint8_t *out = static_cast<uint8_t *>(out_all) + bucket_first * pps * 16;
  const uint32_t *pos = pos_all + bucket_first;
  const float *mu = mu_all ? mu_all + bucket_first : nullptr;
  const uint32_t n_pieces = J * pps;
  const uint32_t stride = gridDim.x * kThreads * kUnroll;
  for (uint32_t base = blockIdx.x * kThreads * kUnroll + threadIdx.x; base < n_pieces; base += stride) {
    u32x4 d[kUnroll];
    uint32_t dst[kUnroll];
    float m[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const uint32_t c = base + i * kThreads;
      if (c < n_pieces) {
        const uint32_t sg = c / pps;
        d[i] = gld<u32x4>(x + (uint64_t)c * 16);
        dst[i] = gld<uint32_t>(pos + sg) * pps + c % pps;
        m[i] = mu ? gld<float>(mu + sg) : 0.0f;
      }
    }
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const uint32_t c = base + i * kThreads;
      if (c < n_pieces) {
        const uint32_t w[4] = {d[i].x, d[i].y, d[i].z, d[i].w};
        uint32_t r[4];
        if constexpr (sizeof(LT) == 4) {
#pragma unroll
          for (int k = 0; k < 4; ++k) r[k] = f2u(u2f(w[k]) - m[i]);
        } else {
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const uint32_t lo = bf16_rne(u2f(w[k] << 16) - m[i]);
            const uint32_t hi = bf16_rne(u2f(w[k] & 0xFFFF0000u) - m[i]);
            r[k] = (lo & 0xFFFFu) | (hi << 16);
          }
        }
        gst<u32x4>(out + (uint64_t)dst[i] * 16, u32x4{r[0], r[1], r[2], r[3]});
      }
    }
  }
}

__global__ void __launch_bounds__(kThreads) k_restore(const float *sum_all, const uint32_t *pos_all, const float *mu_all,
                                                      float n, uint32_t J, float *out_all) {
  constexpr uint32_t pps = kSG * 4 / 16;
  const uint64_t bucket_first = (uint64_t)blockIdx.y * J;
  const uint8_t *sum = reinterpret_cast<const uint8_t *>(sum_all) + bucket_first * pps * 16;
  uint8_t *out = reinterpret_cast<uint8_t *>(out_all) + bucket_first * pps * 16;
  const uint32_t *pos = pos_all + bucket_first;
  const float *mu = mu_all ? mu_all + bucket_first : nullptr;
  const uint32_t n_pieces = J * pps;
  const uint32_t stride = gridDim.x * kThreads * kUnroll;
  for (uint32_t base = blockIdx.x * kThreads * kUnroll + threadIdx.x; base < n_pieces; base += stride) {
    f32x4 d[kUnroll];
    float back[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const uint32_t c = base + i * kThreads;
      if (c < n_pieces) {
        const uint32_t sg = c / pps;
        const uint32_t src = gld<uint32_t>(pos + sg) * pps + c % pps;
        d[i] = gld<f32x4>(sum + (uint64_t)src * 16);
        back[i] = mu ? n * gld<float>(mu + sg) : 0.0f;
      }
    }
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const uint32_t c = base + i * kThreads;
      if (c < n_pieces) {
        f32x4 o;
        o.x = d[i].x + back[i]; o.y = d[i].y + back[i]; o.z = d[i].z + back[i]; o.w = d[i].w + back[i];
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

dq_status launched() { return hipGetLastError() == hipSuccess ? DQ_OK : DQ_EHIP; }

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
                      uint8_t *widths, uint32_t *pos, uint32_t *counts, void *hip_stream) {
  if (n_sg_per_bucket == 0 || n_buckets == 0) return DQ_OK;
  if (!F || !widths || !pos || !counts) return DQ_EINVAL;
  if (max_code_bits < 2ull * n_sg_per_bucket) return DQ_EINVAL;  // fewer than 2 code bits per coordinate
  if (!aligned(F, 4) || !aligned(pos, 4) || !aligned(counts, 4)) return DQ_EALIGN;
  hipStream_t s = (hipStream_t)hip_stream;
  if (n_sg_per_bucket <= (uint32_t)kRegs * kAllocThreads)
    hipLaunchKernelGGL(k_allocate<true>, dim3(n_buckets), dim3(kAllocThreads), 0, s, F, n_sg_per_bucket, max_code_bits,
                       widths, pos, counts);
  else
    hipLaunchKernelGGL(k_allocate<false>, dim3(n_buckets), dim3(kAllocThreads), 0, s, F, n_sg_per_bucket, max_code_bits,
                       widths, pos, counts);
  return launched();
}

dq_status dq_reorder(const void *x, dq_dtype dtype, const uint32_t *pos, const float *mu_or_null,
                     uint32_t n_sg_per_bucket, uint32_t n_buckets, void *out, void *hip_stream) {
  if (n_sg_per_bucket == 0 || n_buckets == 0) return DQ_OK;
  if (!x || !pos || !out || x == out || (dtype != DQ_F32 && dtype != DQ_BF16)) return DQ_EINVAL;
  if (n_sg_per_bucket > (1u << 24) || n_buckets > 65535u) return DQ_EUNSUPPORTED;
  if (!aligned(x, 16) || !aligned(out, 16) || !aligned(pos, 4) || !aligned(mu_or_null, 4)) return DQ_EALIGN;
  const uint64_t pieces = (uint64_t)n_sg_per_bucket * (dtype == DQ_F32 ? 64 : 32);
  const uint32_t blocks = stream_blocks((uint64_t)kThreads * kUnroll, pieces, n_buckets);
  hipStream_t s = (hipStream_t)hip_stream;
  if (dtype == DQ_F32)
    hipLaunchKernelGGL(k_reorder<float>, dim3(blocks, n_buckets), dim3(kThreads), 0, s, x, pos, mu_or_null, n_sg_per_bucket, out);
  else
    hipLaunchKernelGGL(k_reorder<uint16_t>, dim3(blocks, n_buckets), dim3(kThreads), 0, s, x, pos, mu_or_null, n_sg_per_bucket, out);
  return launched();
}

dq_status dq_restore(const float *sum, const uint32_t *pos, const float *mu_or_null, uint32_t n_workers,
                     uint32_t n_sg_per_bucket, uint32_t n_buckets, float *out, void *hip_stream) {
  if (n_sg_per_bucket == 0 || n_buckets == 0) return DQ_OK;
  if (!sum || !pos || !out || sum == out || n_workers == 0) return DQ_EINVAL;
  if (n_sg_per_bucket > (1u << 24) || n_buckets > 65535u) return DQ_EUNSUPPORTED;
  if (!aligned(sum, 16) || !aligned(out, 16) || !aligned(pos, 4) || !aligned(mu_or_null, 4)) return DQ_EALIGN;
  const uint32_t blocks = stream_blocks((uint64_t)kThreads * kUnroll, (uint64_t)n_sg_per_bucket * 64, n_buckets);
  hipLaunchKernelGGL(k_restore, dim3(blocks, n_buckets), dim3(kThreads), 0, (hipStream_t)hip_stream, sum, pos, mu_or_null,
                     (float)n_workers, n_sg_per_bucket, out);
  return launched();
}

}  // extern "C"
