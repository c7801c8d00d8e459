// DynamiQ hot-path kernels for gfx950: compress, decompress-accumulate-recompress (DAR)
// and decompress(+accumulate)  (paper Section 3.3 for the quantizer, Section 3.4 "Fused
// kernels" / Section 4 for which node runs which kernel).
//
// Mapping.  One lane owns one group of 16 entries; a DPP row of 16 lanes is one super-group
// (SG), so the group maximum is in-lane and the SG maximum is four row-rotate DPP steps; a
// wave64 processes 4 SGs per tile and a run of consecutive tiles per launch.  Codes travel as
// one 32/64/128-bit access per lane (2/4/8-bit widths), the local slice as 128-bit accesses.
// Level tables live in LDS from byte 0 on (a block copies only the widths it meets):
//   dec[byte]      the 8/b signed levels (+-T[r]) one byte of packed codes holds  -> decode
//   lut[q]         {T[rc+1], rc} for q = round(x' * 2^m): rc is the level index at the
//                  lower edge of the bin, and bins are narrower than any gap, so the
//                  level at or below x' is rc or rc+1 -- one compare settles it
//   tab[r]         {T[r], D[r]}                                                    -> rounding
// The stochastic rounding follows the division-free form  T + u*D < x'  with
// u = (pi + gamma)/n built from one Philox byte per entry (Section 3.3 "Correlated rounding").
// The per-SG random numbers (group-scale bytes, shared permutation) of up to 8 tiles are
// drawn by ONE wave-wide Philox call (each lane a different counter) and parked in LDS; a block
// with few tiles draws for all its waves at once.  A chunk may end in a run of 16-bit
// super-groups (raw bf16 values, Section 3.2): those tiles only add and round.
// Three options ride on the job: per-super-group means taken off the local entries in fp32 where
// they enter (Section 3.1), the local super-groups gathered from the original tensor through an
// index (the reorder of Section 3.5 done by addressing), and, for decompress, every super-group
// stored to its original place with the mean added back (the restore of Section 3.4, fused in).
//
// All arithmetic that decides a code is IEEE binary32 with explicit fused multiply-adds
// only where written (this file is compiled with -ffp-contract=off and correctly rounded
// division), so the results do not depend on the launch shape.
#include "dq_device.h"

namespace dq {
namespace {

struct NoLocal {};
constexpr int kBatch = 8;  // tiles whose per-SG random numbers one wave-wide draw covers

__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }

// LDS accesses by byte address (the tables are addressed with folded constants)
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const uint32_t lds_u32;
typedef __attribute__((address_space(3))) const u32x2 lds_u2;
typedef __attribute__((address_space(3))) const u32x4 lds_u4;
typedef __attribute__((address_space(3))) u32x4 lds_w4;
__device__ __forceinline__ uint32_t lds_ld1(uint32_t a) { return *reinterpret_cast<lds_u32 *>(a); }
__device__ __forceinline__ u32x2 lds_ld2(uint32_t a) { return *reinterpret_cast<lds_u2 *>(a); }
__device__ __forceinline__ u32x4 lds_ld4(uint32_t a) { return *reinterpret_cast<lds_u4 *>(a); }
__device__ __forceinline__ void lds_st4(uint32_t a, u32x4 v) { *reinterpret_cast<lds_w4 *>(a) = v; }
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) f32x4 lds_f4;
__device__ __forceinline__ void lds_stf4(uint32_t a, f32x4 v) { *reinterpret_cast<lds_f4 *>(a) = v; }
__device__ __forceinline__ f32x4 lds_ldf4(uint32_t a) { return *reinterpret_cast<const lds_f4 *>(a); }

// Global-memory accesses through explicit address-space-1 pointers.  The job's pointers reach
// the kernel inside a struct, where the compiler would otherwise treat them as generic and
// emit FLAT instructions; those also count on the LDS counter, so every wait for a table
// lookup would wait for the outstanding global loads and stores as well.
template <typename T>
__device__ __forceinline__ T gld(const void *p) {
  return *(const __attribute__((address_space(1))) T *)p;
}
template <typename T>
__device__ __forceinline__ void gst(void *p, T v) {
  *(__attribute__((address_space(1))) T *)p = v;
}
__device__ __forceinline__ uint4 gld16(const void *p) {
  const u32x4 t = gld<u32x4>(p);
  return make_uint4(t.x, t.y, t.z, t.w);
}

// ---- Philox4x32-10 (Salmon et al., SC'11): counter-based, so every lane draws its numbers
// from (global group index, round, stream, rank) alone.
struct U4 {
  uint32_t x, y, z, w;
};

// a ^ b ^ c in one instruction (three-input bitwise operation, truth table 0x96)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                            uint32_t k1) {
#pragma unroll
  for (int i = 0; i < 10; ++i) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t a = xor3((uint32_t)(p1 >> 32), c1, k0);
    const uint32_t b = xor3((uint32_t)(p0 >> 32), c3, k1);
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
// (the operands are magnitudes, so the order of their bit patterns is the order of the values)
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ float row_max16(float m) {
  uint32_t x = f2u(m);
  x = max(x, dpp_u<0x128>(x));  // row_ror:8
  x = max(x, dpp_u<0x124>(x));  // row_ror:4
  x = max(x, dpp_u<0x122>(x));  // row_ror:2
  x = max(x, dpp_u<0x121>(x));  // row_ror:1
  return u2f(x);
}

template <int B>
struct Width;
template <>
struct Width<2> { static constexpr int words = 1; };
template <>
struct Width<4> { static constexpr int words = 2; };
template <>
struct Width<8> { static constexpr int words = 4; };

// LDS byte addresses of the tables.  The blob sits at LDS byte 0 (these kernels have dynamic LDS
// only), so the fixed-size tables are compile-time constants that the compiler folds into the
// offset field of the LDS instructions; only the two search tables are found through parameters.
constexpr uint32_t kLds0 = 0;
constexpr uint32_t kRec0 = kLds0 + kOffRec * 4;
template <int B>
__device__ __forceinline__ constexpr uint32_t dec_addr() {
  return kLds0 + (B == 2 ? kOffDec2 : (B == 4 ? kOffDec4 : kOffDec8)) * 4;
}
template <int B>
__device__ __forceinline__ constexpr uint32_t tab_addr() {
  return kLds0 + (B == 4 ? kOffTab4 : kOffTab8) * 4;
}
template <int B>
__device__ __forceinline__ uint32_t lut_addr(const Params &P) {
  if constexpr (B == 4) return kLds0 + kOffLut4 * 4;
  else return kLds0 + P.off_lut8 * 4;
}

// Where a tile (index t in the job's concatenated 2-, 4-, 8-, 16-bit tile sequence) sits.
struct TilePos {
  uint32_t seg_first;   // position in the chunk of the first SG of the tile's width
  uint32_t n_seg;       // SGs of that width in the chunk
  uint32_t tile_first;  // first SG of the tile inside the segment
  int wi;
};
__device__ __forceinline__ TilePos locate(const Job &job, uint32_t t) {
  const uint32_t n0 = job.n_sg[0], n1 = job.n_sg[1], n2 = job.n_sg[2], n3 = job.n_sg[3];
  const uint32_t t0 = (n0 + kWaveSGs - 1) / kWaveSGs, t1 = (n1 + kWaveSGs - 1) / kWaveSGs,
                 t2 = (n2 + kWaveSGs - 1) / kWaveSGs;
  if (t < t0) return TilePos{0, n0, t * kWaveSGs, 0};
  if (t < t0 + t1) return TilePos{n0, n1, (t - t0) * kWaveSGs, 1};
  if (t < t0 + t1 + t2) return TilePos{n0 + n1, n2, (t - t0 - t1) * kWaveSGs, 2};
  return TilePos{n0 + n1 + n2, n3, (t - t0 - t1 - t2) * kWaveSGs, 3};
}

// Wave-uniform addresses of a tile: 64-bit bases once per tile (scalar registers), so that
// every lane only adds a small 32-bit offset.
template <int B>
struct TileBase {
  size_t code_off, gs_off, sf_off;  // byte offsets inside a packed buffer
  size_t first_entry;               // first entry of the tile inside the chunk
  uint32_t last_row;                // rows 0..last_row hold a super-group
  uint64_t G0;                      // global index of the tile's first super-group
  __device__ __forceinline__ TileBase(const Job &job, const TilePos pos) {
    const size_t n0 = job.n_sg[0], n1 = job.n_sg[1], n2 = job.n_sg[2], n3 = job.n_sg[3];
    const size_t c16 = 64 * n0 + 128 * n1 + 256 * n2;  // the raw 16-bit values follow the codes
    const size_t gs0 = c16 + 512 * n3;                  // then the scales of the coded SGs (2, 4, 8 bits)
    const size_t sg0 = (size_t)pos.seg_first + pos.tile_first;  // position in the chunk
    code_off = (B == 2 ? 0 : (B == 4 ? 64 * n0 : (B == 8 ? 64 * n0 + 128 * n1 : c16))) + (size_t)pos.tile_first * (32 * B);
    gs_off = gs0 + sg0 * 16;
    sf_off = gs0 + 16 * (n0 + n1 + n2) + sg0 * 2;
    first_entry = sg0 * kSG;
    last_row = min((uint32_t)kWaveSGs - 1, pos.n_seg - 1 - pos.tile_first);
    G0 = job.first_sg + sg0;
  }
};

// sf_SG/255 and 255/sf_SG for a bf16 sf_SG without a division: the quotient of the 8-bit
// significand comes from a 128-entry table of correctly rounded values and the exponent is
// added on the bit pattern.  Scaling by a power of two commutes with rounding in the normal
// range, so these are exactly the IEEE quotients (encoders never store scales below 2^-100).
__device__ __forceinline__ float sf_over_255(uint32_t sfb, uint32_t rec0) {
  const uint32_t q = lds_ld1(rec0 + (sfb & 0x7Fu) * 8);
  return sfb ? u2f(q + (((sfb >> 7) - 127u) << 23)) : 0.0f;
}
__device__ __forceinline__ float c255_over_sf(uint32_t sfb, uint32_t rec0) {
  const uint32_t q = lds_ld1(rec0 + (sfb & 0x7Fu) * 8 + 4);
  return sfb ? u2f(q - (((sfb >> 7) - 127u) << 23)) : 0.0f;
}

// Section 3.1: the mean of a super-group is subtracted from the local entries in fp32 where they
// enter (one operation per entry on the widened value).  job.mu holds one mean per super-group
// of the chunk, or is null.
__device__ __forceinline__ float local_mean(const Job &job, size_t first_entry, uint32_t row) {
  return job.mu ? gld<float>(job.mu + (first_entry / kSG) + row) : 0.0f;
}
// A lane's 16 local entries (group g of the super-group in row `row` of the tile) as raw 128-bit words.
// Without job.src they sit in the chunk's own order: a wave-uniform base plus a small lane offset.
// With job.src the super-group lives at index src[...] of `local` (the reorder of Section 3.5 done by
// addressing: the kernel gathers whole super-groups, 512 B or 1 KB each, from the original tensor).
// Kernels are built twice: the plain local types know no job.src at all (the compiler would otherwise
// merge the two paths' loads and pay a 64-bit per-lane address on both), the Gathered<> types look at it.
template <typename T>
struct Gathered { T x; };  // same size as T: sizeof(LT) keeps telling fp32 from bf16
template <typename LT>
struct IsGathered { static constexpr bool value = false; };
template <typename T>
struct IsGathered<Gathered<T>> { static constexpr bool value = true; };

template <typename LT>
__device__ __forceinline__ void load_local(const Job &job, size_t first_entry, uint32_t row, uint32_t g,
                                           uint4 (&loc)[sizeof(LT) == 4 ? 4 : 2]) {
  constexpr int kWords = sizeof(LT) == 4 ? 4 : 2;  // 128-bit words per group
  constexpr size_t kSgWords = kSG * sizeof(LT) / 16;
  const uint4 *base = static_cast<const uint4 *>(job.local);
  if constexpr (IsGathered<LT>::value) {
    if (job.src) {
      const size_t sg = gld<uint32_t>(job.src + first_entry / kSG + row);
      const uint4 *p = base + sg * kSgWords + g * kWords;
#pragma unroll
      for (int i = 0; i < kWords; ++i) loc[i] = gld16(p + i);
      return;
    }
  }
  const uint4 *p = base + (first_entry / kSG) * kSgWords + (row * 16 + g) * kWords;
#pragma unroll
  for (int i = 0; i < kWords; ++i) loc[i] = gld16(p + i);
}
template <typename LT>
__device__ __forceinline__ void widen_local(const uint4 (&loc)[sizeof(LT) == 4 ? 4 : 2], float (&v)[16]) {
  if constexpr (sizeof(LT) == 4) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[4 * i] = u2f(loc[i].x); v[4 * i + 1] = u2f(loc[i].y);
      v[4 * i + 2] = u2f(loc[i].z); v[4 * i + 3] = u2f(loc[i].w);
    }
  } else {  // bf16 widens exactly
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t w[4] = {loc[i].x, loc[i].y, loc[i].z, loc[i].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[8 * i + 2 * j] = u2f(w[j] << 16);
        v[8 * i + 2 * j + 1] = u2f(w[j] & 0xFFFF0000u);
      }
    }
  }
}
__device__ __forceinline__ void subtract_mean(const Job &job, float mu, float (&v)[16]) {
  if (job.mu) {
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = v[k] - mu;
  }
}

// What one lane fetches for one tile of compress / DAR: raw words only.
template <int B, Kind KIND, typename LT>
struct Fetch {
  uint4 loc[sizeof(LT) == 4 ? 4 : 2];  // the lane's 16 local entries
  float mu;                            // the mean to take off them (if the job has means)
  uint32_t cw[B / 2];                  // DAR: their incoming codes
  uint32_t rg_in, sf_in;               // DAR: incoming group scale (u8) and SG scale (bf16 pattern)
};

template <int B, Kind KIND, typename LT, bool MU>
__device__ __forceinline__ Fetch<B, KIND, LT> fetch(const Job &job, const TilePos pos) {
  const TileBase<B> tb(job, pos);
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t rowc = min(lane >> 4, tb.last_row);  // idle rows redo the last SG and store nothing
  const uint32_t lg = rowc * 16 + (lane & 15u);       // group index inside the tile
  Fetch<B, KIND, LT> f;
  if constexpr (KIND == kDar) {  // the incoming words first: with job.src the local loads wait for an index
    const uint8_t *cp = job.in + tb.code_off + lg * (2 * B);
    if constexpr (B == 2) {
      f.cw[0] = gld<uint32_t>(cp);
    } else if constexpr (B == 4) {
      const u32x2 t = gld<u32x2>(cp);
      f.cw[0] = t.x; f.cw[1] = t.y;
    } else {
      const u32x4 t = gld<u32x4>(cp);
      f.cw[0] = t.x; f.cw[1] = t.y; f.cw[2] = t.z; f.cw[3] = t.w;
    }
    f.rg_in = gld<uint8_t>(job.in + tb.gs_off + lg);
    f.sf_in = gld<uint16_t>(job.in + tb.sf_off + rowc * 2);
  }
  if constexpr (MU) f.mu = local_mean(job, tb.first_entry, rowc);
  else f.mu = 0.0f;
  load_local<LT>(job, tb.first_entry, rowc, lane & 15u, f.loc);
  return f;
}

// One wave tile of compress / DAR after the fetch: up to 4 super-groups of width B.
//   stage    : LDS byte address of this tile's 8 parked draws (row r: [2r] = permutation
//              stream, [2r+1] = group-scale stream), 16 bytes each
//   ahead    : called once the tile's loaded data is used up, before the per-entry work: from there the
//              next tile's loads have the longest time to arrive without holding two tiles' data at once
template <int B, Kind KIND, typename LT, bool MU, typename Ahead>
__device__ __forceinline__ void compute(const Job &job, const Params &P, uint32_t stage,
                                        const TilePos pos, const Fetch<B, KIND, LT> &f, Ahead ahead) {
  using W = Width<B>;
  static_assert(KIND != kDecompress, "decompress has its own tile function");
  const TileBase<B> tb(job, pos);
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t g = lane & 15u;
  const uint32_t row = lane >> 4;
  const bool active = row <= tb.last_row;
  const uint32_t rowc = min(row, tb.last_row);
  const uint32_t lg = rowc * 16 + g;
  constexpr uint32_t rec0 = kRec0;

  // ------------------------------------------------------------------ random numbers
  // (first: they need nothing from memory, so a wave that still waits for its tile has them done;
  // the empty asm ties the tile's first use to them, or the scheduler would sink them below the wait)
  const uint64_t gi = (tb.G0 + rowc) * 16 + g;  // global group index
  // stream 0: one byte per entry, private to the worker
  const U4 gam = philox4x32_10((uint32_t)gi, (uint32_t)(gi >> 32), P.round, job.rank & 0xFFFFu, P.key0, P.key1);
  // parked per-SG draws: this worker's slot pi_rank of the shared permutation (group g of the
  // super-group uses pi_rank + g mod n); byte g of the private stream -> this group's scale dither
  const uint32_t slot0 = lds_ld1(stage + rowc * 32);
  const uint32_t sc_word = lds_ld1(stage + rowc * 32 + 16 + (g >> 2) * 4);
  const uint32_t scale_byte = (sc_word >> (8 * (g & 3u))) & 0xFFu;
  uint32_t slot = slot0 + g;  // below n + 16
  slot = (P.n_mask != 0xFFFFFFFFu) ? (slot & P.n_mask) : (slot % P.n_workers);
  const float o_pi = ((float)slot + (1.0f / 512.0f)) * P.inv_n;

  uint4 loc[sizeof(LT) == 4 ? 4 : 2];
#pragma unroll
  for (int i = 0; i < (sizeof(LT) == 4 ? 4 : 2); ++i) loc[i] = f.loc[i];
  asm volatile("" : "+v"(loc[0].x) : "v"(gam.x), "v"(gam.y), "v"(gam.z), "v"(gam.w), "v"(o_pi), "v"(scale_byte));
  float v[16];
  widen_local<LT>(loc, v);
  if constexpr (MU) {
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = v[k] - f.mu;
  }

  if constexpr (KIND == kDar) {
    // decode: sf_G = r_G * (sf_SG / 255); estimate = +-T[r] * sf_G, accumulated by one fma
    const float sfg = (float)f.rg_in * sf_over_255(f.sf_in, rec0);
    constexpr uint32_t dec0 = dec_addr<B>();
#pragma unroll
    for (int j = 0; j < 2 * B; ++j) {  // one table entry per code byte
      const uint32_t byte = (f.cw[j >> 2] >> (8 * (j & 3))) & 0xFFu;
      if constexpr (B == 2) {
        const u32x4 e = lds_ld4(dec0 + byte * 16);
        v[4 * j] = __builtin_fmaf(u2f(e.x), sfg, v[4 * j]);
        v[4 * j + 1] = __builtin_fmaf(u2f(e.y), sfg, v[4 * j + 1]);
        v[4 * j + 2] = __builtin_fmaf(u2f(e.z), sfg, v[4 * j + 2]);
        v[4 * j + 3] = __builtin_fmaf(u2f(e.w), sfg, v[4 * j + 3]);
      } else if constexpr (B == 4) {
        const u32x2 e = lds_ld2(dec0 + byte * 8);
        v[2 * j] = __builtin_fmaf(u2f(e.x), sfg, v[2 * j]);
        v[2 * j + 1] = __builtin_fmaf(u2f(e.y), sfg, v[2 * j + 1]);
      } else {
        v[j] = __builtin_fmaf(u2f(lds_ld1(dec0 + byte * 4)), sfg, v[j]);
      }
    }
  }

  // ------------------------------------------------------------------ scales
  float m = 0.0f;
#pragma unroll
  for (int k = 0; k < 16; ++k) m = fmaxf(m, fabsf(v[k]));
  const float M = row_max16(m);
  uint32_t sfb = f2u(M) >> 16;
  sfb += (f2u(M) & 0xFFFFu) ? 1u : 0u;  // smallest bf16 >= M
  if (sfb < 0x0D80u) sfb = 0;           // below 2^-100: the SG is encoded as zero
  const float cs = c255_over_sf(sfb, rec0);
  const float ts = fminf(m * cs, 255.0f);
  const float fl = floorf(ts);
  const float us = ((float)scale_byte + 0.5f) * (1.0f / 256.0f);
  const uint32_t rg = sfb ? (uint32_t)fl + ((us < ts - fl) ? 1u : 0u) : 0u;
  // a group whose scale rounds to zero keeps only its signs; its entries are not normalised
  const float inv = rg ? 1.0f / m : 0.0f;

  ahead();

  // ------------------------------------------------------------------ entries
  // x' = |v| * inv needs no clamp: |v| <= m and inv is the correctly rounded 1/m, so the exact
  // product is at most 1 + 2^-24, which rounds to 1.  The product is taken with v's sign (xs): the
  // magnitude serves the search and the rounding through source modifiers, the top bit is the
  // code's sign bit (for inv = 0 the product is a zero with v's sign).
  // The code words grow from the top: entry 15 first, each step shifts the word by one code and
  // appends sign and level index, so the lowest entry of a word ends in its low bits.  A group
  // whose scale rounded to zero has inv = 0, hence x' = 0 and level 0 throughout: only signs remain.
  uint32_t ow[W::words];
#pragma unroll
  for (int i = 0; i < W::words; ++i) ow[i] = 0;
  const uint32_t gw[4] = {gam.x, gam.y, gam.z, gam.w};
  if constexpr (B == 2) {
    // levels {0,1}: T + u*D = u, so the level bit is [u < x'] -- the sign bit of u - x' (the
    // difference of two different binary32 numbers is never zero)
#pragma unroll
    for (int k = 15; k >= 0; --k) {
      const float xs = v[k] * inv;
      const uint32_t byte = (gw[k >> 2] >> (8 * (k & 3))) & 0xFFu;
      const float u = __builtin_fmaf((float)byte, P.s_n, o_pi);
      const float d = u - fabsf(xs);
      ow[0] = __builtin_amdgcn_alignbit(ow[0], f2u(xs), 31);  // (word << 1) | sign
      ow[0] = __builtin_amdgcn_alignbit(ow[0], f2u(d), 31);   // (word << 1) | level
    }
  } else {
    const float magic = P.magic[B == 4 ? 1 : 2];
    // byte address of lut[q] is lut0 + 8*q with q = bits(x + magic) - bits(magic)
    uint32_t lut_k = lut_addr<B>(P) - (f2u(magic) << 3);
    asm("" : "+s"(lut_k));  // one scalar: (bits << 3) + lut_k is then a single shift-add per entry
    constexpr uint32_t tab0 = tab_addr<B>();
    constexpr int per_word = 32 / B;
#pragma unroll
    for (int k = 15; k >= 0; --k) {
      const float xs = v[k] * inv;
      const float x = fabsf(xs);
      const uint32_t byte = (gw[k >> 2] >> (8 * (k & 3))) & 0xFFu;
      const float u = __builtin_fmaf((float)byte, P.s_n, o_pi);
      const u32x2 e = lds_ld2((f2u(x + magic) << 3) + lut_k);
      uint32_t rlo = e.y + ((x >= u2f(e.x)) ? 1u : 0u);
      asm("" : "+v"(rlo));  // keep r = rlo + [..] below from being re-derived as e.y + [..] + [..]
      const u32x2 td = lds_ld2(tab0 + rlo * 8);
      const uint32_t up = (__builtin_fmaf(u, u2f(td.y), u2f(td.x)) < x) ? 1u : 0u;
      const uint32_t w = __builtin_amdgcn_alignbit(ow[k / per_word], f2u(xs), 31);  // (word << 1) | sign
      ow[k / per_word] = (w << (B - 1)) + rlo + up;  // level index r_lo + [rounded up] <= R: no carry into the sign
    }
  }

  // ------------------------------------------------------------------ store
  if (active) {
    uint8_t *out = static_cast<uint8_t *>(job.out);
    uint8_t *cp = out + tb.code_off + lg * (2 * B);
    if constexpr (B == 2) {
      gst<uint32_t>(cp, ow[0]);
    } else if constexpr (B == 4) {
      gst<u32x2>(cp, u32x2{ow[0], ow[1]});
    } else {
      gst<u32x4>(cp, u32x4{ow[0], ow[1], ow[2], ow[3]});
    }
    gst<uint8_t>(out + tb.gs_off + lg, (uint8_t)rg);
    if (g == 0) gst<uint16_t>(out + tb.sf_off + rowc * 2, (uint16_t)sfb);
  }
}

// A wave tile's 4 KB of fp32 results, v[16] per lane (lane = group), written through the wave's
// LDS area so that every store instruction covers 1 KB of contiguous memory: lane l parks its 4
// float4 at slots 4l..4l+3 (slot index xor-ed with bits 2-3 of l so that the 16 lanes of a pass hit
// different banks); store round r then reads slot r*64 + lane = float4 number r*64 + lane of the tile.
__device__ __forceinline__ void store_tile_f32(const Job &job, const Params &P, float (&v)[16], uint32_t xpose,
                                               size_t first_entry, uint32_t last_row) {
  const uint32_t lane = threadIdx.x & 63u;
  const size_t sg0 = first_entry / kSG;  // the tile's first super-group inside the chunk
  if (job.back) {
    // Section 3.4, last paragraph: the mean comes back, n times (the sum of n workers' entries lost it n times)
    const float back = (float)P.n_workers * gld<float>(job.back + sg0 + min(lane >> 4, last_row));
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = v[k] + back;
  }
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (uint32_t i = 0; i < 4; ++i)
    lds_stf4(xpose + lane * 64 + ((i ^ ((lane >> 2) & 3u)) * 16), f32x4{v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]});
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  float *out = static_cast<float *>(job.out);
#pragma unroll
  for (uint32_t r = 0; r < (uint32_t)kWaveSGs; ++r) {
    if (r > last_row) break;
    const uint32_t slot = r * 64 + lane, w = slot >> 2, c = slot & 3u;
    const f32x4 o = lds_ldf4(xpose + w * 64 + ((c ^ ((w >> 2) & 3u)) * 16));
    // row r is one super-group, 1 KB: at its place in the chunk, or where job.dest sends it
    const size_t sg = job.dest ? (size_t)gld<uint32_t>(job.dest + sg0 + r) : sg0 + r;
    gst<f32x4>(reinterpret_cast<float4 *>(out + sg * kSG) + lane, o);
  }
  __builtin_amdgcn_wave_barrier();
}

// One wave tile of decompress(+accumulate).  Lanes fetch and decode like the DAR tile (a lane
// owns a group of 16 entries, few wide loads), then the 4 KB of fp32 results are transposed
// through a per-wave LDS area so that every store instruction writes 1 KB of contiguous memory.
//   xpose : LDS byte address of this wave's 4 KB transpose area
template <int B, typename LT>
__device__ __forceinline__ void tile_da(const Job &job, const Params &P, uint32_t xpose,
                                        const TilePos pos) {
  using W = Width<B>;
  constexpr bool kHasLocal = !__is_same(LT, NoLocal);
  const TileBase<B> tb(job, pos);
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t rowc = min(lane >> 4, tb.last_row);
  const uint32_t lg = rowc * 16 + (lane & 15u);
  constexpr uint32_t rec0 = kRec0;
  constexpr uint32_t dec0 = dec_addr<B>();

  // the incoming words first: with job.src the local loads wait for an index
  uint32_t cw[W::words];
  const uint8_t *cp = job.in + tb.code_off + lg * (2 * B);
  if constexpr (B == 2) {
    cw[0] = gld<uint32_t>(cp);
  } else if constexpr (B == 4) {
    const u32x2 t = gld<u32x2>(cp);
    cw[0] = t.x; cw[1] = t.y;
  } else {
    const u32x4 t = gld<u32x4>(cp);
    cw[0] = t.x; cw[1] = t.y; cw[2] = t.z; cw[3] = t.w;
  }
  const uint32_t rg_in = gld<uint8_t>(job.in + tb.gs_off + lg);
  const uint32_t sf_in = gld<uint16_t>(job.in + tb.sf_off + rowc * 2);
  float v[16];
  float mu = 0.0f;
  if constexpr (kHasLocal) {
    uint4 loc[sizeof(LT) == 4 ? 4 : 2];
    mu = local_mean(job, tb.first_entry, rowc);
    load_local<LT>(job, tb.first_entry, rowc, lane & 15u, loc);
    widen_local<LT>(loc, v);
  }
  const float sfg = (float)rg_in * sf_over_255(sf_in, rec0);
  // after every load of the tile has been issued: the branch would otherwise hold the later loads back
  if constexpr (kHasLocal) subtract_mean(job, mu, v);
#pragma unroll
  for (int j = 0; j < 2 * B; ++j) {  // one table entry per code byte
    const uint32_t byte = (cw[j >> 2] >> (8 * (j & 3))) & 0xFFu;
    float t[4];
    constexpr int per = 8 / B;
    if constexpr (B == 2) {
      const u32x4 e = lds_ld4(dec0 + byte * 16);
      t[0] = u2f(e.x); t[1] = u2f(e.y); t[2] = u2f(e.z); t[3] = u2f(e.w);
    } else if constexpr (B == 4) {
      const u32x2 e = lds_ld2(dec0 + byte * 8);
      t[0] = u2f(e.x); t[1] = u2f(e.y);
    } else {
      t[0] = u2f(lds_ld1(dec0 + byte * 4));
    }
#pragma unroll
    for (int k = 0; k < per; ++k) {
      if constexpr (kHasLocal) v[per * j + k] = __builtin_fmaf(t[k], sfg, v[per * j + k]);
      else v[per * j + k] = t[k] * sfg;
    }
  }
  store_tile_f32(job, P, v, xpose, tb.first_entry, tb.last_row);
}

// Decompress-accumulate over `len` consecutive tiles of width B: the tile's operands are those of a DAR
// hop (fetch<.., kDar, ..>); the next tile is requested before the current one's transpose and stores.
template <int B, typename LT, bool MU>
__device__ __forceinline__ void run_tiles_da(const Job &job, const Params &P, uint32_t xpose, TilePos pos, uint32_t len) {
  constexpr uint32_t rec0 = kRec0;
  constexpr uint32_t dec0 = dec_addr<B>();
  Fetch<B, kDar, LT> f = fetch<B, kDar, LT, MU>(job, pos);
  for (uint32_t i = 0; i < len; ++i) {
    const TileBase<B> tb(job, pos);
    float v[16];
    widen_local<LT>(f.loc, v);
    if constexpr (MU) {
#pragma unroll
      for (int k = 0; k < 16; ++k) v[k] = v[k] - f.mu;
    }
    const float sfg = (float)f.rg_in * sf_over_255(f.sf_in, rec0);
#pragma unroll
    for (int j = 0; j < 2 * B; ++j) {  // one table entry per code byte
      const uint32_t byte = (f.cw[j >> 2] >> (8 * (j & 3))) & 0xFFu;
      if constexpr (B == 2) {
        const u32x4 e = lds_ld4(dec0 + byte * 16);
        v[4 * j] = __builtin_fmaf(u2f(e.x), sfg, v[4 * j]);
        v[4 * j + 1] = __builtin_fmaf(u2f(e.y), sfg, v[4 * j + 1]);
        v[4 * j + 2] = __builtin_fmaf(u2f(e.z), sfg, v[4 * j + 2]);
        v[4 * j + 3] = __builtin_fmaf(u2f(e.w), sfg, v[4 * j + 3]);
      } else if constexpr (B == 4) {
        const u32x2 e = lds_ld2(dec0 + byte * 8);
        v[2 * j] = __builtin_fmaf(u2f(e.x), sfg, v[2 * j]);
        v[2 * j + 1] = __builtin_fmaf(u2f(e.y), sfg, v[2 * j + 1]);
      } else {
        v[j] = __builtin_fmaf(u2f(lds_ld1(dec0 + byte * 4)), sfg, v[j]);
      }
    }
    TilePos pos_next = pos;
    pos_next.tile_first += kWaveSGs;
    if (i + 1 < len) f = fetch<B, kDar, LT, MU>(job, pos_next);
    store_tile_f32(job, P, v, xpose, tb.first_entry, tb.last_row);
    pos = pos_next;
  }
}

// One wave tile of uncompressed (16-bit) super-groups: the packed values are raw bf16
// ("16 bits corresponds to uncompressed values", Section 3.2).  Compress rounds the local entries
// to bf16 (nearest even); a DAR hop adds the local entry to the widened incoming value in fp32
// and rounds the sum back; decompress widens (and adds).  No scales, no random numbers.
__device__ __forceinline__ uint32_t bf16_rne_pair(float lo, float hi) {
  const uint32_t a = f2u(lo), b = f2u(hi);
  const uint32_t ra = (a + 0x7FFFu + ((a >> 16) & 1u)) >> 16;
  const uint32_t rb = (b + 0x7FFFu + ((b >> 16) & 1u)) & 0xFFFF0000u;
  return ra | rb;
}

template <Kind KIND, typename LT>
__device__ __forceinline__ void tile16(const Job &job, const Params &P, uint32_t xpose, const TilePos pos) {
  constexpr bool kHasLocal = !__is_same(LT, NoLocal);
  const TileBase<16> tb(job, pos);
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t row = lane >> 4;
  const uint32_t rowc = min(row, tb.last_row);
  const uint32_t lg = rowc * 16 + (lane & 15u);
  uint4 in[2];
  if constexpr (KIND != kCompress) {  // the incoming words first: with job.src the local loads wait for an index
    const uint4 *p = reinterpret_cast<const uint4 *>(job.in + tb.code_off) + lg * 2;
    in[0] = gld16(p);
    in[1] = gld16(p + 1);
  }
  float v[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) v[k] = 0.0f;
  float mu = 0.0f;
  if constexpr (kHasLocal) {
    uint4 loc[sizeof(LT) == 4 ? 4 : 2];
    mu = local_mean(job, tb.first_entry, rowc);
    load_local<LT>(job, tb.first_entry, rowc, lane & 15u, loc);
    widen_local<LT>(loc, v);
  }
  if constexpr (kHasLocal) subtract_mean(job, mu, v);  // after every load of the tile has been issued
  if constexpr (KIND != kCompress) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint4 x = in[i];
      const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[8 * i + 2 * j] = u2f(w[j] << 16) + v[8 * i + 2 * j];
        v[8 * i + 2 * j + 1] = u2f(w[j] & 0xFFFF0000u) + v[8 * i + 2 * j + 1];
      }
    }
  }
  if constexpr (KIND == kDecompress) {
    store_tile_f32(job, P, v, xpose, tb.first_entry, tb.last_row);
  } else if (row <= tb.last_row) {
    uint8_t *dst = static_cast<uint8_t *>(job.out) + tb.code_off + lg * 32;
#pragma unroll
    for (int i = 0; i < 2; ++i)
      gst<u32x4>(dst + 16 * i, u32x4{bf16_rne_pair(v[8 * i], v[8 * i + 1]), bf16_rne_pair(v[8 * i + 2], v[8 * i + 3]),
                                     bf16_rne_pair(v[8 * i + 4], v[8 * i + 5]), bf16_rne_pair(v[8 * i + 6], v[8 * i + 7])});
  }
}

// `len` consecutive tiles of width B starting at `pos` (their parked draws 128 bytes apart).
template <int B, Kind KIND, typename LT, bool MU>
__device__ __forceinline__ void run_tiles(const Job &job, const Params &P, uint32_t stage, TilePos pos,
                                          uint32_t len) {
  // The next tile of the run is requested from inside the current one (see compute's `ahead`): with five waves
  // per SIMD a wave's own wait for its tile is no longer covered by the others (measured: 3-7 % on the 25 MB
  // and the 100-bucket configurations, nothing on the largest launches).
  Fetch<B, KIND, LT> f = fetch<B, KIND, LT, MU>(job, pos);
  for (uint32_t i = 0; i < len; ++i) {
    Fetch<B, KIND, LT> next = f;
    TilePos pos_next = pos;
    pos_next.tile_first += kWaveSGs;
    const bool more = i + 1 < len;
    compute<B, KIND, LT, MU>(job, P, stage + i * 128, pos, f, [&] {
      if (more) next = fetch<B, KIND, LT, MU>(job, pos_next);
    });
    f = next;
    pos = pos_next;
  }
}

// The shared random permutation pi of 0..n-1 (Section 3.3 "Correlated rounding") at one worker
// index, from the four words of the super-group's shared draw: three rounds of
//   y <- reverse_k(((w_t | 1) * y + (w_t >> 16)) mod 2^k),  k = ceil(log2 n)
// (odd multiply, add and bit reversal are bijections of the k-bit integers), walked again while
// the value is not below n, then rotated by floor(w3 * n / 2^32) so that every worker's slot is
// uniform.  Evaluated once per super-group and job (the rank is the job's), never per entry.
__device__ __forceinline__ uint32_t perm_slot(const U4 &d, const Params &P, uint32_t rank) {
  const uint32_t k = P.perm_bits, mask = (1u << k) - 1u, back = (32u - k) & 31u;
  const uint32_t w[3] = {d.x, d.y, d.z};
  auto rounds = [&](uint32_t y) {
#pragma unroll
    for (int t = 0; t < 3; ++t) y = __brev(((w[t] | 1u) * y + (w[t] >> 16)) & mask) >> back;
    return y;
  };
  uint32_t y = rounds(rank);
  if (P.n_mask == 0xFFFFFFFFu)  // n is not a power of two: some k-bit values lie outside 0..n-1
    while (y >= P.n_workers) y = rounds(y);  // ends: the walk is a cycle through `rank` < n
  const uint32_t s = y + __umulhi(d.w, P.n_workers);
  return s >= P.n_workers ? s - P.n_workers : s;
}

// Per-SG draws of `nb` <= 8 consecutive tiles starting at tile `t_first`, made by one wave-wide
// Philox call and parked at `area` (128 bytes per tile: row r at [32r] this worker's slot of the
// shared permutation, at [32r+16] the worker's group-scale stream).  Lane l draws for tile l/8, row (l%8)/2.
__device__ __forceinline__ void park_draws(const Job &job, const Params &P, uint32_t t_first, uint32_t nb,
                                           uint32_t area) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t j = min(lane >> 3, nb - 1);
  const TilePos p = locate(job, t_first + j);
  const uint32_t sgw = min(p.tile_first + ((lane >> 1) & 3u), p.n_seg - 1);
  const uint64_t G = job.first_sg + p.seg_first + sgw;
  const uint32_t c3 = (lane & 1u) ? ((1u << 16) | (job.rank & 0xFFFFu)) : ((2u << 16) | 0xFFFFu);
  const U4 d = philox4x32_10((uint32_t)G, (uint32_t)(G >> 32), P.round, c3, P.key0, P.key1);
  // even lanes hold the shared draw: they park the slot it gives this job's worker in word 0
  const uint32_t w0 = (lane & 1u) ? d.x : perm_slot(d, P, job.rank);
  lds_st4(area + lane * 16, u32x4{w0, d.y, d.z, d.w});
}

// Tiles [t_first, t_first + nb) of the job, whose draws are parked from `area` on.
template <Kind KIND, typename LT>
__device__ __forceinline__ void run_range(const Job &job, const Params &P, uint32_t area,
                                          uint32_t t_first, uint32_t nb) {
  for (uint32_t j = 0; j < nb;) {
    const TilePos p = locate(job, t_first + j);
    const uint32_t left = (p.n_seg - p.tile_first + kWaveSGs - 1) / kWaveSGs;  // tiles to the segment's end
    const uint32_t len = min(nb - j, left);
    const uint32_t stage = area + j * 128;
    // two builds of the tile loop, with and without means: a branch on job.mu inside a tile makes the
    // path without means wait, at the branch's join, for the loads issued before it
    if (job.mu) {
      if (p.wi == 0) run_tiles<2, KIND, LT, true>(job, P, stage, p, len);
      else if (p.wi == 1) run_tiles<4, KIND, LT, true>(job, P, stage, p, len);
      else if (p.wi == 2) run_tiles<8, KIND, LT, true>(job, P, stage, p, len);
    } else {
      if (p.wi == 0) run_tiles<2, KIND, LT, false>(job, P, stage, p, len);
      else if (p.wi == 1) run_tiles<4, KIND, LT, false>(job, P, stage, p, len);
      else if (p.wi == 2) run_tiles<8, KIND, LT, false>(job, P, stage, p, len);
    }
    if (p.wi > 2) {
      TilePos q = p;
      for (uint32_t i = 0; i < len; ++i, q.tile_first += kWaveSGs) tile16<KIND, LT>(job, P, 0u, q);
    }
    j += len;
  }
}

// Decompress(+accumulate) over the job's tiles [w_lo, w_hi): tile by tile without a local slice, in
// runs of one width (the next tile requested ahead) with one.
template <typename LT>
__device__ __forceinline__ void da_range(const Job &job, const Params &P, uint32_t xpose, uint32_t w_lo, uint32_t w_hi) {
  if constexpr (__is_same(LT, NoLocal)) {
    for (uint32_t t = w_lo; t < w_hi; ++t) {
      const TilePos p = locate(job, t);
      if (p.wi == 0) tile_da<2, LT>(job, P, xpose, p);
      else if (p.wi == 1) tile_da<4, LT>(job, P, xpose, p);
      else if (p.wi == 2) tile_da<8, LT>(job, P, xpose, p);
      else tile16<kDecompress, LT>(job, P, xpose, p);
    }
  } else {
    for (uint32_t t = w_lo; t < w_hi;) {  // runs of one width, as in run_range
      const TilePos p = locate(job, t);
      const uint32_t left = (p.n_seg - p.tile_first + kWaveSGs - 1) / kWaveSGs;
      const uint32_t len = min(w_hi - t, left);
      if (job.mu) {
        if (p.wi == 0) run_tiles_da<2, LT, true>(job, P, xpose, p, len);
        else if (p.wi == 1) run_tiles_da<4, LT, true>(job, P, xpose, p, len);
        else if (p.wi == 2) run_tiles_da<8, LT, true>(job, P, xpose, p, len);
      } else {
        if (p.wi == 0) run_tiles_da<2, LT, false>(job, P, xpose, p, len);
        else if (p.wi == 1) run_tiles_da<4, LT, false>(job, P, xpose, p, len);
        else if (p.wi == 2) run_tiles_da<8, LT, false>(job, P, xpose, p, len);
      }
      if (p.wi > 2) {
        TilePos q = p;
        for (uint32_t i = 0; i < len; ++i, q.tile_first += kWaveSGs) tile16<kDecompress, LT>(job, P, xpose, q);
      }
      t += len;
    }
  }
}

// The job's tiles are split evenly over all waves of the grid row (4 * gridDim.x waves):
// wave w takes [w*T/W, (w+1)*T/W).  The launcher sizes the grid to what the GPU holds at
// once, so a wave lives for the whole launch and the table copy is paid once.
template <Kind KIND, typename LT>
__device__ __forceinline__ void run_job(const Job &job, const Params &P) {
  extern __shared__ uint4 lds_raw[];
  uint32_t *lds = reinterpret_cast<uint32_t *>(lds_raw);
  const uint32_t n0 = job.n_sg[0], n1 = job.n_sg[1], n2 = job.n_sg[2];
  const uint32_t t0 = (n0 + kWaveSGs - 1) / kWaveSGs, t1 = (n1 + kWaveSGs - 1) / kWaveSGs,
                 t2 = (n2 + kWaveSGs - 1) / kWaveSGs, t3 = (job.n_sg[3] + kWaveSGs - 1) / kWaveSGs;
  const uint32_t total = t0 + t1 + t2 + t3;
  // even split of the tiles over the grid's waves in 32-bit arithmetic: wave v takes q tiles
  // from v*q + min(v, r), one more if v < r (q, r = quotient and remainder of tiles by waves)
  const uint32_t n_waves = gridDim.x * kBlockWaves;
  const uint32_t q = total / n_waves, r = total - q * n_waves;
  const uint32_t bw = blockIdx.x * kBlockWaves;
  const uint32_t b_lo = bw * q + min(bw, r);
  const uint32_t b_hi = (bw + kBlockWaves) * q + min(bw + kBlockWaves, r);
  if (b_lo >= b_hi) return;
  constexpr uint32_t lds0 = kLds0;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t wv = bw + wave;
  const uint32_t w_lo = wv * q + min(wv, r);
  const uint32_t w_hi = w_lo + q + (wv < r ? 1u : 0u);
  // parking area for per-SG draws: 1 KB (8 tiles) per wave, the four areas contiguous
  // (decompress needs no search tables: its blocks leave them out and are small enough for six per CU)
  const uint32_t park0 = lds0 + (KIND == kDecompress ? kOffLut4 : P.blob_dwords) * 4;
  // a block with at most 32 tiles makes all its draws up front, 8 tiles per wave-wide call,
  // instead of one call per wave (waves of a small job hold only a tile or two each)
  const bool block_draws = KIND != kDecompress && (b_hi - b_lo) <= 8u * kBlockWaves;

  // copy the common tables and the table ranges of the widths this block meets; the first
  // 16 bytes per thread of every range are requested together (one round trip, not six)
  const bool meets[4] = {b_lo < t0, b_lo < t0 + t1 && b_hi > t0, b_lo < t0 + t1 + t2 && b_hi > t0 + t1, true};
  constexpr int kEarly = kRanges;
  uint4 first[kEarly];
  bool need[kRanges], has[kEarly];
#pragma unroll
  for (int r = 0; r < kRanges; ++r)
    need[r] = meets[P.range_width[r] & 3u] && !(KIND == kDecompress && P.range_lo[r] >= kOffLut4);
#pragma unroll
  for (int r = 0; r < kEarly; ++r) {
    const uint32_t i = P.range_lo[r] + threadIdx.x * 4;
    has[r] = need[r] && i < P.range_hi[r];
    if (has[r]) first[r] = gld16(&P.blob[i]);
  }
  if constexpr (KIND != kDecompress) {
    if (block_draws && 8u * wave < b_hi - b_lo)
      park_draws(job, P, b_lo + 8u * wave, min(8u, b_hi - b_lo - 8u * wave), park0 + wave * 1024);
  }
#pragma unroll
  for (int r = 0; r < kEarly; ++r)
    if (has[r]) *reinterpret_cast<uint4 *>(&lds[P.range_lo[r] + threadIdx.x * 4]) = first[r];
#pragma unroll
  for (int r = 0; r < kRanges; ++r)
    if (need[r])
      for (uint32_t i = P.range_lo[r] + ((r < kEarly ? kBlockThreads : 0) + threadIdx.x) * 4; i < P.range_hi[r]; i += kBlockThreads * 4)
        *reinterpret_cast<uint4 *>(&lds[i]) = gld16(&P.blob[i]);
  __syncthreads();

  if constexpr (KIND == kDecompress) {
    // per-wave transpose area: 64 lanes x 64 bytes
    const uint32_t xpose = park0 + wave * (64 * 64);
    da_range<LT>(job, P, xpose, w_lo, w_hi);
  } else if (block_draws) {
    run_range<KIND, LT>(job, P, park0 + (w_lo - b_lo) * 128, w_lo, w_hi - w_lo);
  } else {
    const uint32_t area = park0 + wave * 1024;
    for (uint32_t tb = w_lo; tb < w_hi; tb += kBatch) {
      const uint32_t nb = min((uint32_t)kBatch, w_hi - tb);
      park_draws(job, P, tb, nb, area);
      __builtin_amdgcn_wave_barrier();
      run_range<KIND, LT>(job, P, area, tb, nb);
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// Five blocks of four waves are resident per CU (the launcher's grid): at most 96 vector registers (the kernels
// with fp32 locals use 82-88 since a tile's successor is requested from inside the tile, the others at most 80).
template <Kind KIND, typename LT>
__global__ __launch_bounds__(kBlockThreads) void k_one(Job job, Params P) {
  run_job<KIND, LT>(job, P);
}
template <Kind KIND, typename LT>
__global__ __launch_bounds__(kBlockThreads) void k_batch(const Job *jobs, Params P) {
  const Job job = jobs[blockIdx.y];
  run_job<KIND, LT>(job, P);
}
// Launches of thousands of jobs of at most kBatch tiles each (a replay of thousands of simulated workers:
// a tile or two per chunk): one job per WAVE, so that a block's table copy and its place on a CU serve
// four jobs instead of one wave's worth of one.
template <Kind KIND, typename LT>
__global__ __launch_bounds__(kBlockThreads) void k_batch_small(const Job *jobs, uint32_t n_jobs, Params P) {
  extern __shared__ uint4 lds_raw[];
  uint32_t *lds = reinterpret_cast<uint32_t *>(lds_raw);
  // every table range: the block's four jobs may meet any width (decompress never needs the search tables)
#pragma unroll
  for (int r = 0; r < kRanges; ++r)
    if (!(KIND == kDecompress && P.range_lo[r] >= kOffLut4))
      for (uint32_t i = P.range_lo[r] + threadIdx.x * 4; i < P.range_hi[r]; i += kBlockThreads * 4)
        *reinterpret_cast<uint4 *>(&lds[i]) = gld16(&P.blob[i]);
  __syncthreads();
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t j = __builtin_amdgcn_readfirstlane(blockIdx.x * kBlockWaves + wave);
  if (j >= n_jobs) return;
  const Job job = jobs[j];
  const uint32_t tiles = (job.n_sg[0] + kWaveSGs - 1) / kWaveSGs + (job.n_sg[1] + kWaveSGs - 1) / kWaveSGs +
                         (job.n_sg[2] + kWaveSGs - 1) / kWaveSGs + (job.n_sg[3] + kWaveSGs - 1) / kWaveSGs;
  if (tiles == 0) return;
  const uint32_t park0 = kLds0 + (KIND == kDecompress ? kOffLut4 : P.blob_dwords) * 4;
  if constexpr (KIND == kDecompress) {
    da_range<LT>(job, P, park0 + wave * (64 * 64), 0u, tiles);
  } else {
    const uint32_t area = park0 + wave * 1024;
    park_draws(job, P, 0u, tiles, area);
    __builtin_amdgcn_wave_barrier();
    run_range<KIND, LT>(job, P, area, 0u, tiles);
  }
}

// Copy of a packed block in 16-byte words; the bytes from `valid` on (the padding at the block's end,
// which the codec kernels never write) are put down as zero.
__global__ void __launch_bounds__(256) k_wire_copy(const uint4 *src, uint4 *dst, uint64_t words, uint64_t valid) {
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (uint64_t)gridDim.x * 256) {
    uint4 w = src[i];
    if ((i + 1) * 16 > valid) {
      uint32_t x[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint64_t at = i * 16 + 4 * k;  // first byte of this dword
        const uint32_t keep = at >= valid ? 0u : (valid - at >= 4 ? 0xFFFFFFFFu : (1u << (8 * (uint32_t)(valid - at))) - 1u);
        x[k] &= keep;
      }
      w = uint4{x[0], x[1], x[2], x[3]};
    }
    dst[i] = w;
  }
}

uint32_t job_tiles(const Job &j) {
  return (j.n_sg[0] + kWaveSGs - 1) / kWaveSGs + (j.n_sg[1] + kWaveSGs - 1) / kWaveSGs +
         (j.n_sg[2] + kWaveSGs - 1) / kWaveSGs + (j.n_sg[3] + kWaveSGs - 1) / kWaveSGs;
}

// Grid shape: `grid_blocks` (what the GPU holds at once: CUs x blocks per CU, fixed when the
// context is made) shared between the jobs of the launch (one block holds 4 waves; a wave
// then walks its share of the job's tiles).
uint32_t blocks_per_job(uint32_t max_tiles, uint32_t n_jobs, uint32_t grid_blocks) {
  uint32_t blocks = (grid_blocks + n_jobs - 1) / n_jobs;
  const uint32_t needed = (max_tiles + kBlockWaves - 1) / kBlockWaves;
  if (blocks > needed) blocks = needed;
  return blocks < 1 ? 1 : blocks;
}

// blob + per-wave area: 1 KB of parked draws (compress, DAR) or 4 KB for the transpose (decompress)
size_t lds_bytes(const Params &p, Kind kind) {
  return kind == kDecompress ? (size_t)kOffLut4 * 4 + kBlockWaves * 64 * 64 : (size_t)p.blob_dwords * 4 + kBlockWaves * 64 * 16;
}

template <Kind KIND, typename LT>
hipError_t go_one(const Job &job, Params p, uint32_t grid_blocks, hipStream_t s) {
  const uint32_t tiles = job_tiles(job);
  if (tiles == 0) return hipSuccess;
  const uint32_t blocks = blocks_per_job(tiles, 1, grid_blocks);
  hipLaunchKernelGGL((k_one<KIND, LT>), dim3(blocks), dim3(kBlockThreads), lds_bytes(p, KIND), s, job, p);
  return hipGetLastError();
}
template <Kind KIND, typename LT>
hipError_t go_batch(const Job *jobs, uint32_t n_jobs, uint32_t max_tiles, uint64_t total_tiles, Params p,
                    uint32_t grid_blocks, hipStream_t s) {
  if (n_jobs == 0 || max_tiles == 0) return hipSuccess;
  (void)total_tiles;
  if (max_tiles <= (uint32_t)kBatch && n_jobs >= grid_blocks) {  // so many small jobs that a block per job would queue up
    hipLaunchKernelGGL((k_batch_small<KIND, LT>), dim3((n_jobs + kBlockWaves - 1) / kBlockWaves), dim3(kBlockThreads),
                       lds_bytes(p, KIND), s, jobs, n_jobs, p);
    return hipGetLastError();
  }
  const uint32_t blocks = blocks_per_job(max_tiles, n_jobs, grid_blocks);
  // the grid's y dimension (one row per job) holds at most 65,535 rows: more jobs take more launches
  for (uint32_t first = 0; first < n_jobs; first += kMaxGridRows) {
    const uint32_t rows = n_jobs - first < kMaxGridRows ? n_jobs - first : kMaxGridRows;
    hipLaunchKernelGGL((k_batch<KIND, LT>), dim3(blocks, rows), dim3(kBlockThreads), lds_bytes(p, KIND), s, jobs + first, p);
  }
  return hipGetLastError();
}

}  // namespace

// LT for a local of `dtype`, gathered through job.src or not
#define DQ_DISPATCH_LOCAL(CALL, KINDV)                                                        \
  (gather ? (f32 ? CALL<KINDV, Gathered<float>> ARGS : CALL<KINDV, Gathered<uint16_t>> ARGS) \
          : (f32 ? CALL<KINDV, float> ARGS : CALL<KINDV, uint16_t> ARGS))

hipError_t launch_one(Kind kind, dq_dtype dtype, bool has_local, const Job &job, const Params &p, uint32_t grid_blocks,
                      hipStream_t s) {
  const bool f32 = dtype == DQ_F32, gather = job.src != nullptr;
#define ARGS (job, p, grid_blocks, s)
  switch (kind) {
    case kCompress: return DQ_DISPATCH_LOCAL(go_one, kCompress);
    case kDar: return DQ_DISPATCH_LOCAL(go_one, kDar);
    default:
      if (!has_local) return go_one<kDecompress, NoLocal>(job, p, grid_blocks, s);
      return DQ_DISPATCH_LOCAL(go_one, kDecompress);
  }
#undef ARGS
}

hipError_t launch_batch(Kind kind, dq_dtype dtype, bool has_local, bool gather, const Job *jobs, uint32_t n_jobs,
                        uint32_t max_tiles, uint64_t total_tiles, const Params &p, uint32_t grid_blocks, hipStream_t s) {
  const bool f32 = dtype == DQ_F32;
#define ARGS (jobs, n_jobs, max_tiles, total_tiles, p, grid_blocks, s)
  switch (kind) {
    case kCompress: return DQ_DISPATCH_LOCAL(go_batch, kCompress);
    case kDar: return DQ_DISPATCH_LOCAL(go_batch, kDar);
    default:
      if (!has_local) return go_batch<kDecompress, NoLocal>(jobs, n_jobs, max_tiles, total_tiles, p, grid_blocks, s);
      return DQ_DISPATCH_LOCAL(go_batch, kDecompress);
  }
#undef ARGS
}
#undef DQ_DISPATCH_LOCAL

namespace {
template <typename K>
hipError_t add_static_lds(K kernel, size_t *bytes) {
  hipFuncAttributes attr;
  const hipError_t e = hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(kernel));
  if (e == hipSuccess && attr.sharedSizeBytes > *bytes) *bytes = attr.sharedSizeBytes;
  return e;
}
template <Kind KIND, typename LT>
hipError_t add_static_lds_of(size_t *bytes) {
  const hipError_t e = add_static_lds(k_one<KIND, LT>, bytes);
  return e != hipSuccess ? e : add_static_lds(k_batch<KIND, LT>, bytes);
}
}  // namespace

hipError_t static_lds_bytes(size_t *bytes) {
  *bytes = 0;
  hipError_t e = add_static_lds_of<kDecompress, NoLocal>(bytes);
#define DQ_ONE_KIND(KINDV)                                                             \
  if (e == hipSuccess) e = add_static_lds_of<KINDV, float>(bytes);                     \
  if (e == hipSuccess) e = add_static_lds_of<KINDV, uint16_t>(bytes);                  \
  if (e == hipSuccess) e = add_static_lds_of<KINDV, Gathered<float>>(bytes);           \
  if (e == hipSuccess) e = add_static_lds_of<KINDV, Gathered<uint16_t>>(bytes);
  DQ_ONE_KIND(kCompress)
  DQ_ONE_KIND(kDar)
  DQ_ONE_KIND(kDecompress)
#undef DQ_ONE_KIND
  return e;
}

hipError_t wire_copy(void *dst, const void *src, size_t bytes, size_t valid, hipStream_t s) {
  const uint64_t words = bytes / 16;
  if (words == 0) return hipSuccess;
  const uint64_t want = (words + 1023) / 1024;  // four words per thread
  const uint32_t blocks = (uint32_t)(want < 2048 ? want : 2048);
  hipLaunchKernelGGL(k_wire_copy, dim3(blocks), dim3(256), 0, s, static_cast<const uint4 *>(src), static_cast<uint4 *>(dst),
                     words, (uint64_t)valid);
  return hipGetLastError();
}

}  // namespace dq
