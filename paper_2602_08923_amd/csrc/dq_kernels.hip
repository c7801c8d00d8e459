// DynamiQ hot-path kernels for gfx950: compress, decompress-accumulate-recompress (DAR)
// and decompress(+accumulate)  (paper Section 3.3 for the quantizer, Section 3.4 "Fused
// kernels" / Section 4 for which node runs which kernel).
//
// Mapping.  One lane owns one group of 16 entries; a DPP row of 16 lanes is one super-group
// (SG), so the group maximum is in-lane and the SG maximum is four row-rotate DPP steps; a
// wave64 processes 4 SGs per tile.  Codes travel as one 32/64/128-bit access per lane
// (2/4/8-bit widths), the local slice as 128-bit accesses.  Level tables live in LDS:
//   dec[code]      signed level  (+-T[r])                                  -> decode
//   lut[q]         {T[rc+1], rc} for q = round(x' * 2^m): rc is the level index at the
//                  lower edge of the bin, and bins are narrower than any gap, so the
//                  level at or below x' is rc or rc+1 -- one compare settles it
//   tab[r]         {T[r], D[r]}                                            -> rounding
// The stochastic rounding follows the division-free form  T + u*D < x'  with
// u = (pi + gamma)/n built from one Philox byte per entry (Section 3.3 "Correlated rounding").
//
// All arithmetic that decides a code is IEEE binary32 with explicit fused multiply-adds
// only where written (this file is compiled with -ffp-contract=off and correctly rounded
// division), so the results do not depend on the launch shape.
#include "dq_device.h"

namespace dq {
namespace {

struct NoLocal {};

__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }

// ---- Philox4x32-10 (Salmon et al., SC'11): counter-based, so every lane draws its numbers
// from (global group index, round, stream, rank) alone.
struct U4 {
  uint32_t x, y, z, w;
};

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                            uint32_t k1) {
#pragma unroll
  for (int i = 0; i < 10; ++i) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t a = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t b = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = a;
    c2 = b;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return U4{c0, c1, c2, c3};
}

// ---- max over the 16 lanes of a DPP row, result in every lane of the row
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return u2f((uint32_t)__builtin_amdgcn_update_dpp(0, (int)f2u(x), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float row_max16(float x) {
  x = fmaxf(x, dpp_f<0x128>(x));  // row_ror:8
  x = fmaxf(x, dpp_f<0x124>(x));  // row_ror:4
  x = fmaxf(x, dpp_f<0x122>(x));  // row_ror:2
  x = fmaxf(x, dpp_f<0x121>(x));  // row_ror:1
  return x;
}

template <int B>
struct Width;
template <>
struct Width<2> { static constexpr int wi = 0, words = 1, R = 1; };
template <>
struct Width<4> { static constexpr int wi = 1, words = 2, R = 7; };
template <>
struct Width<8> { static constexpr int wi = 2, words = 4, R = 127; };

template <typename LT>
__device__ __forceinline__ void load_local(const void *base, size_t first, float (&loc)[16]) {
  if constexpr (sizeof(LT) == 4) {  // fp32: 4 x 128 bit
    const float4 *p = reinterpret_cast<const float4 *>(static_cast<const float *>(base) + first);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float4 t = p[i];
      loc[4 * i] = t.x; loc[4 * i + 1] = t.y; loc[4 * i + 2] = t.z; loc[4 * i + 3] = t.w;
    }
  } else {  // bf16: 2 x 128 bit, widened exactly
    const uint4 *p = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + first);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint4 t = p[i];
      const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        loc[8 * i + 2 * j] = u2f(w[j] << 16);
        loc[8 * i + 2 * j + 1] = u2f(w[j] & 0xFFFF0000u);
      }
    }
  }
}

// One wave tile: up to 4 super-groups of width B.
//   seg_first : position in the chunk of the first SG of this width
//   n_seg     : SGs of this width in the chunk (>= 1)
//   tile_first: first SG of the tile inside the segment
//   code_off  : byte offset of this width's code array inside a packed buffer
template <int B, Kind KIND, typename LT>
__device__ __forceinline__ void tile(const Job &job, const Params &P, const uint32_t *lds, uint32_t seg_first,
                                     uint32_t n_seg, uint32_t tile_first, size_t code_off) {
  using W = Width<B>;
  constexpr bool kHasLocal = !__is_same(LT, NoLocal);
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t g = lane & 15u;
  const uint32_t sgw_raw = tile_first + (lane >> 4);
  const bool active = sgw_raw < n_seg;
  const uint32_t sgw = active ? sgw_raw : n_seg - 1;  // idle rows redo the last SG and store nothing
  const uint32_t sgj = seg_first + sgw;               // position in the chunk
  const size_t n_all = (size_t)job.n_sg[0] + job.n_sg[1] + job.n_sg[2];
  const size_t gs_off = 64 * (size_t)job.n_sg[0] + 128 * (size_t)job.n_sg[1] + 256 * (size_t)job.n_sg[2];
  const size_t sf_off = gs_off + 16 * n_all;
  const size_t code_at = code_off + ((size_t)sgw * 16 + g) * (2 * B);

  float v[16];
  // ------------------------------------------------------------------ gather inputs
  if constexpr (kHasLocal) load_local<LT>(job.local, (size_t)sgj * kSG + g * kGroup, v);

  if constexpr (KIND != kCompress) {
    uint32_t cw[W::words];
    if constexpr (B == 2) {
      cw[0] = *reinterpret_cast<const uint32_t *>(job.in + code_at);
    } else if constexpr (B == 4) {
      const uint2 t = *reinterpret_cast<const uint2 *>(job.in + code_at);
      cw[0] = t.x; cw[1] = t.y;
    } else {
      const uint4 t = *reinterpret_cast<const uint4 *>(job.in + code_at);
      cw[0] = t.x; cw[1] = t.y; cw[2] = t.z; cw[3] = t.w;
    }
    const uint32_t rg_in = job.in[gs_off + (size_t)sgj * 16 + g];
    const uint32_t sf_in = *reinterpret_cast<const uint16_t *>(job.in + sf_off + (size_t)sgj * 2);
    // decode: sf_G = r_G * (sf_SG / 255); estimate = +-T[r] * sf_G, accumulated by one fma
    const float step = u2f(sf_in << 16) / 255.0f;
    const float sfg = (float)rg_in * step;
    const uint32_t *dec = lds + P.off_dec[W::wi];
    constexpr int per_word = 32 / B;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const uint32_t code = (cw[k / per_word] >> ((k % per_word) * B)) & ((1u << B) - 1u);
      const float t = u2f(dec[code]);
      if constexpr (kHasLocal) v[k] = __builtin_fmaf(t, sfg, v[k]);
      else v[k] = t * sfg;
    }
  }

  if constexpr (KIND == kDecompress) {
    if (active) {
      float4 *o = reinterpret_cast<float4 *>(static_cast<float *>(job.out) + (size_t)sgj * kSG + g * kGroup);
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = make_float4(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]);
    }
    return;
  } else {
    // ---------------------------------------------------------------- random numbers
    const uint64_t G = job.first_sg + sgj;  // global super-group index
    const uint64_t gi = G * 16 + g;         // global group index
    // stream 0: one byte per entry, private to the worker
    const U4 gam = philox4x32_10((uint32_t)gi, (uint32_t)(gi >> 32), P.round, job.rank & 0xFFFFu, P.key0, P.key1);
    // streams 1 (group-scale bytes, private) and 2 (shared cyclic shift) are per SG: lane 0 of
    // the row draws stream 2, the others draw stream 1, then the row exchanges the words
    const uint32_t c3 = (g == 0) ? ((2u << 16) | 0xFFFFu) : ((1u << 16) | (job.rank & 0xFFFFu));
    const U4 sgr = philox4x32_10((uint32_t)G, (uint32_t)(G >> 32), P.round, c3, P.key0, P.key1);
    const uint32_t row0 = lane & ~15u;
    const uint32_t perm_w0 = __shfl(sgr.x, row0);
    // lanes 1..15 all hold the stream-1 words; group g's scale byte sits in word g>>2
    const uint32_t w_mine = (g >> 2) == 0 ? sgr.x : (g >> 2) == 1 ? sgr.y : (g >> 2) == 2 ? sgr.z : sgr.w;
    // lane 0 did not draw stream 1: it needs word 0 of a neighbour
    const uint32_t w_nb = __shfl(sgr.x, row0 + 1);
    const uint32_t sc_word = (g == 0) ? w_nb : w_mine;
    const uint32_t scale_byte = (sc_word >> (8 * (g & 3u))) & 0xFFu;
    const uint32_t shift = __umulhi(perm_w0, P.n_workers);
    uint32_t slot = job.rank + shift + g;
    slot = (P.n_mask != 0xFFFFFFFFu) ? (slot & P.n_mask) : (slot % P.n_workers);
    const float o_pi = ((float)slot + (1.0f / 512.0f)) * P.inv_n;

    // ---------------------------------------------------------------- scales
    float m = 0.0f;
#pragma unroll
    for (int k = 0; k < 16; ++k) m = fmaxf(m, fabsf(v[k]));
    const float M = row_max16(m);
    uint32_t sfb = f2u(M) >> 16;
    sfb += (f2u(M) & 0xFFFFu) ? 1u : 0u;  // smallest bf16 >= M
    if (sfb < 0x0D80u) sfb = 0;           // below 2^-100: the SG is encoded as zero
    const float sf = u2f(sfb << 16);
    const float cs = sfb ? 255.0f / sf : 0.0f;
    const float t = fminf(m * cs, 255.0f);
    const float fl = floorf(t);
    const float us = ((float)scale_byte + 0.5f) * (1.0f / 256.0f);
    const uint32_t rg = sfb ? (uint32_t)fl + ((us < t - fl) ? 1u : 0u) : 0u;
    const float inv = 1.0f / m;  // unused (and possibly inf) when rg == 0

    // ---------------------------------------------------------------- entries
    uint32_t ow[W::words];
#pragma unroll
    for (int i = 0; i < W::words; ++i) ow[i] = 0;
    const uint32_t gw[4] = {gam.x, gam.y, gam.z, gam.w};
    constexpr int per_word = 32 / B;
    const float magic = P.magic[W::wi];
    const uint2 *lut = reinterpret_cast<const uint2 *>(lds + P.off_lut[W::wi]);
    const uint2 *tab = reinterpret_cast<const uint2 *>(lds + P.off_tab[W::wi]);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const float x = fminf(fabsf(v[k]) * inv, 1.0f);
      const uint32_t byte = (gw[k >> 2] >> (8 * (k & 3))) & 0xFFu;
      const float u = __builtin_fmaf((float)byte, P.s_n, o_pi);
      uint32_t r;
      if constexpr (B == 2) {
        r = (u < x) ? 1u : 0u;  // levels {0,1}: T + u*D = u
      } else {
        const uint32_t q = f2u(x + magic) - f2u(magic);  // round(x * 2^m)
        const uint2 e = lut[q];
        const uint32_t rlo = e.y + ((x >= u2f(e.x)) ? 1u : 0u);
        const uint2 td = tab[rlo];
        r = rlo + ((__builtin_fmaf(u, u2f(td.y), u2f(td.x)) < x) ? 1u : 0u);
      }
      r = rg ? r : 0u;
      const uint32_t code = ((f2u(v[k]) >> 31) << (B - 1)) | r;
      ow[k / per_word] |= code << ((k % per_word) * B);
    }

    // ---------------------------------------------------------------- store
    if (active) {
      uint8_t *out = static_cast<uint8_t *>(job.out);
      if constexpr (B == 2) {
        *reinterpret_cast<uint32_t *>(out + code_at) = ow[0];
      } else if constexpr (B == 4) {
        *reinterpret_cast<uint2 *>(out + code_at) = make_uint2(ow[0], ow[1]);
      } else {
        *reinterpret_cast<uint4 *>(out + code_at) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
      }
      out[gs_off + (size_t)sgj * 16 + g] = (uint8_t)rg;
      if (g == 0) *reinterpret_cast<uint16_t *>(out + sf_off + (size_t)sgj * 2) = (uint16_t)sfb;
    }
  }
}

template <Kind KIND, typename LT>
__device__ __forceinline__ void run_job(const Job &job, const Params &P) {
  extern __shared__ uint32_t lds[];
  for (uint32_t i = threadIdx.x * 4; i < P.blob_dwords; i += kBlockThreads * 4)
    *reinterpret_cast<uint4 *>(&lds[i]) = *reinterpret_cast<const uint4 *>(&P.blob[i]);
  __syncthreads();
  const uint32_t n0 = job.n_sg[0], n1 = job.n_sg[1], n2 = job.n_sg[2];
  const uint32_t t0 = (n0 + kWaveSGs - 1) / kWaveSGs, t1 = (n1 + kWaveSGs - 1) / kWaveSGs,
                 t2 = (n2 + kWaveSGs - 1) / kWaveSGs;
  const uint32_t total = t0 + t1 + t2;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  for (uint32_t t = blockIdx.x * kBlockWaves + wave; t < total; t += gridDim.x * kBlockWaves) {
    if (t < t0) {
      tile<2, KIND, LT>(job, P, lds, 0, n0, t * kWaveSGs, 0);
    } else if (t < t0 + t1) {
      tile<4, KIND, LT>(job, P, lds, n0, n1, (t - t0) * kWaveSGs, 64 * (size_t)n0);
    } else {
      tile<8, KIND, LT>(job, P, lds, n0 + n1, n2, (t - t0 - t1) * kWaveSGs, 64 * (size_t)n0 + 128 * (size_t)n1);
    }
  }
}

template <Kind KIND, typename LT>
__global__ __launch_bounds__(kBlockThreads) void k_one(Job job, Params P) {
  run_job<KIND, LT>(job, P);
}
template <Kind KIND, typename LT>
__global__ __launch_bounds__(kBlockThreads) void k_batch(const Job *jobs, Params P) {
  const Job job = jobs[blockIdx.y];
  run_job<KIND, LT>(job, P);
}

uint32_t job_tiles(const Job &j) {
  return (j.n_sg[0] + kWaveSGs - 1) / kWaveSGs + (j.n_sg[1] + kWaveSGs - 1) / kWaveSGs +
         (j.n_sg[2] + kWaveSGs - 1) / kWaveSGs;
}

template <Kind KIND, typename LT>
hipError_t go_one(const Job &job, const Params &p, uint32_t n_cu, hipStream_t s) {
  const uint32_t tiles = job_tiles(job);
  if (tiles == 0) return hipSuccess;
  uint32_t blocks = (tiles + kBlockWaves - 1) / kBlockWaves;
  const uint32_t cap = n_cu * 8;
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL((k_one<KIND, LT>), dim3(blocks), dim3(kBlockThreads), p.blob_dwords * 4, s, job, p);
  return hipGetLastError();
}
template <Kind KIND, typename LT>
hipError_t go_batch(const Job *jobs, uint32_t n_jobs, uint32_t max_tiles, const Params &p, uint32_t n_cu,
                    hipStream_t s) {
  if (n_jobs == 0 || max_tiles == 0) return hipSuccess;
  uint32_t blocks = (max_tiles + kBlockWaves - 1) / kBlockWaves;
  uint32_t cap = (n_cu * 8 + n_jobs - 1) / n_jobs;
  if (cap < 1) cap = 1;
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL((k_batch<KIND, LT>), dim3(blocks, n_jobs), dim3(kBlockThreads), p.blob_dwords * 4, s, jobs, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_one(Kind kind, dq_dtype dtype, bool has_local, const Job &job, const Params &p, uint32_t n_cu,
                      hipStream_t s) {
  const bool f32 = dtype == DQ_F32;
  switch (kind) {
    case kCompress:
      return f32 ? go_one<kCompress, float>(job, p, n_cu, s) : go_one<kCompress, uint16_t>(job, p, n_cu, s);
    case kDar:
      return f32 ? go_one<kDar, float>(job, p, n_cu, s) : go_one<kDar, uint16_t>(job, p, n_cu, s);
    default:
      if (!has_local) return go_one<kDecompress, NoLocal>(job, p, n_cu, s);
      return f32 ? go_one<kDecompress, float>(job, p, n_cu, s) : go_one<kDecompress, uint16_t>(job, p, n_cu, s);
  }
}

hipError_t launch_batch(Kind kind, dq_dtype dtype, bool has_local, const Job *jobs, uint32_t n_jobs,
                        uint32_t max_tiles, const Params &p, uint32_t n_cu, hipStream_t s) {
  const bool f32 = dtype == DQ_F32;
  switch (kind) {
    case kCompress:
      return f32 ? go_batch<kCompress, float>(jobs, n_jobs, max_tiles, p, n_cu, s)
                 : go_batch<kCompress, uint16_t>(jobs, n_jobs, max_tiles, p, n_cu, s);
    case kDar:
      return f32 ? go_batch<kDar, float>(jobs, n_jobs, max_tiles, p, n_cu, s)
                 : go_batch<kDar, uint16_t>(jobs, n_jobs, max_tiles, p, n_cu, s);
    default:
      if (!has_local) return go_batch<kDecompress, NoLocal>(jobs, n_jobs, max_tiles, p, n_cu, s);
      return f32 ? go_batch<kDecompress, float>(jobs, n_jobs, max_tiles, p, n_cu, s)
                 : go_batch<kDecompress, uint16_t>(jobs, n_jobs, max_tiles, p, n_cu, s);
  }
}

}  // namespace dq
