// OCP Microscaling (MXFP8 E4M3 / MXFP6 E3M2 / MXFP4 E2M1) versions of compress, DAR and
// decompress(+accumulate) -- the comparison codec of the paper's evaluation (Section 5,
// "Baseline compression schemes") run in the same hop loop.  Conversion per the OCP MX v1.0
// specification: shared exponent floor(log2 max|v|) - emax_elem stored as an E8M0 byte,
// elements rounded to nearest-even and clamped to the largest normal.
//
// Mapping: one lane owns one block of 32 entries (its maximum is in-lane); a wave64 covers
// 2048 entries per tile.
#include "dq_device.h"

namespace dq {
namespace {

struct NoLocal {};

__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }

// explicit global (address space 1) accesses: the job's pointers arrive inside a struct and
// would otherwise be treated as generic, i.e. FLAT instructions
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
template <typename T>
__device__ __forceinline__ T gld(const void *p) {
  return *(const __attribute__((address_space(1))) T *)p;
}
template <typename T>
__device__ __forceinline__ void gst(void *p, T v) {
  *(__attribute__((address_space(1))) T *)p = v;
}

typedef __attribute__((address_space(3))) f32x4 lds_f32x4;
__device__ __forceinline__ void lds_put(uint32_t a, f32x4 v) { *reinterpret_cast<lds_f32x4 *>(a) = v; }
__device__ __forceinline__ f32x4 lds_get(uint32_t a) { return *reinterpret_cast<const lds_f32x4 *>(a); }

template <int FMT>
struct Fmt;
template <>
struct Fmt<DQ_MXFP8_E4M3> { static constexpr int emax = 8, cb = 8; };  // largest exponent, code bits
template <>
struct Fmt<DQ_MXFP6_E3M2> { static constexpr int emax = 4, cb = 6; };
template <>
struct Fmt<DQ_MXFP4_E2M1> { static constexpr int emax = 2, cb = 4; };

template <typename LT>
__device__ __forceinline__ void load_local32(const void *base, size_t first, float (&v)[32]) {
  if constexpr (sizeof(LT) == 4) {
    const float4 *p = reinterpret_cast<const float4 *>(static_cast<const float *>(base) + first);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const f32x4 t = gld<f32x4>(p + i);
      v[4 * i] = t.x; v[4 * i + 1] = t.y; v[4 * i + 2] = t.z; v[4 * i + 3] = t.w;
    }
  } else {
    const uint4 *p = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + first);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u32x4 t = gld<u32x4>(p + i);
      const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[8 * i + 2 * j] = u2f(w[j] << 16);
        v[8 * i + 2 * j + 1] = u2f(w[j] & 0xFFFF0000u);
      }
    }
  }
}

// One block of 32 entries per lane, converted by gfx950's scaled conversion instructions
// (V_CVT_SCALEF32_*): packed elements <-> fp32 with the block scale applied in the same
// instruction, round to nearest even.  What measurement against the CPU oracle showed about them:
//   - the scale operand is a binary32 whose exponent FIELD is taken as the E8M0 byte (so the
//     pattern e << 23 is passed, also for e = 0);
//   - the E4M3 narrowing turns overflow into NaN (0x7F) where MX saturates: values are clamped
//     to +-448 * 2^(e-127) first (same result as round-then-saturate); E3M2 and E2M1 saturate;
//   - the instruction set's "fp6" is E2M3; OCP's MXFP6 E3M2 is its "bf6";
//   - the 32-wide 6-bit narrowing interleaves its two 16-entry inputs (a0 b0 a1 b1 ...), the
//     widening returns entries in order.
// Decoded element * scale is exact in binary32 for every code and scale byte, so adding the
// local entry afterwards is the single-rounding fma the conversion rule asks for.
typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x6 __attribute__((ext_vector_type(6)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x32 __attribute__((ext_vector_type(32)));

template <int FMT, Kind KIND, typename LT>
__device__ __forceinline__ void mx_block(const MxJob &job, uint64_t bi, uint64_t n_blocks, bool active, uint32_t xpose) {
  using F = Fmt<FMT>;
  constexpr bool kHasLocal = !__is_same(LT, NoLocal);
  constexpr int cw = F::cb;
  const size_t scale_off = (size_t)n_blocks * (cw * 4);
  const uint64_t bl = active ? bi : n_blocks - 1;  // block whose inputs this lane reads
  float v[32];
  if constexpr (kHasLocal) load_local32<LT>(job.local, (size_t)bl * 32, v);
  if constexpr (KIND != kCompress) {
    uint32_t w[cw];
    const uint8_t *src = job.in + (size_t)bl * (cw * 4);
    if constexpr (cw == 8) {
      const u32x4 a = gld<u32x4>(src), b = gld<u32x4>(src + 16);
      w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
    } else if constexpr (cw == 6) {
      const u32x2 a = gld<u32x2>(src), b = gld<u32x2>(src + 8), c = gld<u32x2>(src + 16);
      w[0] = a.x; w[1] = a.y; w[2] = b.x; w[3] = b.y; w[4] = c.x; w[5] = c.y;
    } else {
      const u32x4 a = gld<u32x4>(src);
      w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
    }
    const uint32_t e = gld<uint8_t>(job.in + scale_off + bl);
    const float X = u2f(e << 23);  // the instruction reads the exponent field as the E8M0 scale
    float d[32];
    if constexpr (cw == 8) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const f32x2 lo = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(w[i], X, false);
        const f32x2 hi = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(w[i], X, true);
        d[4 * i] = lo.x; d[4 * i + 1] = lo.y; d[4 * i + 2] = hi.x; d[4 * i + 3] = hi.y;
      }
    } else if constexpr (cw == 4) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const f32x2 b0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], X, 0);
        const f32x2 b1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], X, 1);
        const f32x2 b2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], X, 2);
        const f32x2 b3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], X, 3);
        d[8 * i] = b0.x; d[8 * i + 1] = b0.y; d[8 * i + 2] = b1.x; d[8 * i + 3] = b1.y;
        d[8 * i + 4] = b2.x; d[8 * i + 5] = b2.y; d[8 * i + 6] = b3.x; d[8 * i + 7] = b3.y;
      }
    } else {
      const f32x32 all = __builtin_amdgcn_cvt_scalef32_pk32_f32_bf6(u32x6{w[0], w[1], w[2], w[3], w[4], w[5]}, X);
#pragma unroll
      for (int k = 0; k < 32; ++k) d[k] = all[k];
    }
#pragma unroll
    for (int k = 0; k < 32; ++k) v[k] = kHasLocal ? d[k] + v[k] : d[k];
  }
  if constexpr (KIND == kDecompress) {
    // The wave's 64 blocks are 8 KB of consecutive output.  Lane l parks its 8 float4 in the
    // wave's LDS area (slot index xor-ed with l % 8 against bank conflicts); round r then
    // stores float4 number 64 r + l of the tile, 1 KB of consecutive memory per instruction.
    const uint32_t lane = threadIdx.x & 63u;
    if (active) {
#pragma unroll
      for (uint32_t c = 0; c < 8; ++c)
        lds_put(xpose + lane * 128 + ((c ^ (lane & 7u)) * 16), f32x4{v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]});
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint64_t tile_first = bi - lane;  // first block of the wave's tile
    float4 *o = reinterpret_cast<float4 *>(static_cast<float *>(job.out) + (size_t)tile_first * 32);
#pragma unroll
    for (uint32_t r = 0; r < 8; ++r) {
      const uint32_t L = r * 64 + lane, w = L >> 3, c = L & 7u;
      if (tile_first + w < n_blocks) gst<f32x4>(o + L, lds_get(xpose + w * 128 + ((c ^ (w & 7u)) * 16)));
    }
    __builtin_amdgcn_wave_barrier();  // the area is reused by the wave's next tile
  } else {
    float m = 0.0f;
#pragma unroll
    for (int k = 0; k < 32; ++k) m = fmaxf(m, fabsf(v[k]));
    int e = (int)(f2u(m) >> 23) - F::emax;
    e = e < 0 ? 0 : (e > 254 ? 254 : e);
    const float X = u2f((uint32_t)e << 23);
    uint32_t ow[cw];
    if constexpr (cw == 8) {
      // the E4M3 conversion turns overflow into NaN; MX saturates: clamp to the largest normal first
      const float top = 448.0f * X;
#pragma unroll
      for (int k = 0; k < 32; ++k) v[k] = __builtin_amdgcn_fmed3f(v[k], -top, top);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        s16x2 r = {0, 0};
        r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, v[4 * i], v[4 * i + 1], X, false);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, v[4 * i + 2], v[4 * i + 3], X, true);
        ow[i] = __builtin_bit_cast(uint32_t, r);
      }
    } else if constexpr (cw == 4) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint32_t r = 0;
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * i], v[8 * i + 1], X, 0);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * i + 2], v[8 * i + 3], X, 1);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * i + 4], v[8 * i + 5], X, 2);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * i + 6], v[8 * i + 7], X, 3);
        ow[i] = r;
      }
    } else {
      f32x16 a, b;
#pragma unroll
      for (int k = 0; k < 16; ++k) { a[k] = v[2 * k]; b[k] = v[2 * k + 1]; }  // the two inputs interleave
      const u32x6 r = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(a, b, X);
#pragma unroll
      for (int i = 0; i < 6; ++i) ow[i] = r[i];
    }
    uint8_t *dst = static_cast<uint8_t *>(job.out) + (size_t)bi * (cw * 4);
    if constexpr (cw == 8) {
      gst<u32x4>(dst, u32x4{ow[0], ow[1], ow[2], ow[3]});
      gst<u32x4>(dst + 16, u32x4{ow[4], ow[5], ow[6], ow[7]});
    } else if constexpr (cw == 6) {
      gst<u32x2>(dst, u32x2{ow[0], ow[1]});
      gst<u32x2>(dst + 8, u32x2{ow[2], ow[3]});
      gst<u32x2>(dst + 16, u32x2{ow[4], ow[5]});
    } else {
      gst<u32x4>(dst, u32x4{ow[0], ow[1], ow[2], ow[3]});
    }
    gst<uint8_t>(static_cast<uint8_t *>(job.out) + scale_off + bi, (uint8_t)e);
  }
}

template <int FMT, Kind KIND, typename LT>
__device__ __forceinline__ void mx_run(const MxJob &job) {
  const uint64_t n_blocks = job.n_entries / 32;
  const uint64_t stride = (uint64_t)gridDim.x * kBlockThreads;
  if constexpr (KIND == kDecompress) {
    // whole waves walk the tiles of 64 blocks together (the stores are a wave-wide transpose);
    // lanes past the end of a ragged last tile redo the last block and store nothing
    __shared__ float4 park[kBlockWaves * 512];  // 8 KB per wave
    const uint32_t xpose = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float4 *)park + (threadIdx.x >> 6) * 8192;
    const uint64_t first = (uint64_t)blockIdx.x * kBlockThreads + (threadIdx.x & ~63u);
    for (uint64_t t0 = first; t0 < n_blocks; t0 += stride) {
      const uint64_t bi = t0 + (threadIdx.x & 63u);
      mx_block<FMT, KIND, LT>(job, bi, n_blocks, bi < n_blocks, xpose);
    }
  } else {
    for (uint64_t bi = (uint64_t)blockIdx.x * kBlockThreads + threadIdx.x; bi < n_blocks; bi += stride)
      mx_block<FMT, KIND, LT>(job, bi, n_blocks, true, 0u);
  }
}

template <int FMT, Kind KIND, typename LT>
__global__ __launch_bounds__(kBlockThreads) void mx_one(MxJob job) {
  mx_run<FMT, KIND, LT>(job);
}
template <int FMT, Kind KIND, typename LT>
__global__ __launch_bounds__(kBlockThreads) void mx_batch(const MxJob *jobs) {
  const MxJob job = jobs[blockIdx.y];
  mx_run<FMT, KIND, LT>(job);
}

template <int FMT, Kind KIND, typename LT>
hipError_t go(const MxJob *one, const MxJob *jobs, uint32_t n_jobs, uint64_t max_entries, uint32_t n_cu, hipStream_t s) {
  const uint64_t blocks_needed = (max_entries / 32 + kBlockThreads - 1) / kBlockThreads;
  if (blocks_needed == 0 || n_jobs == 0) return hipSuccess;
  uint64_t cap = ((uint64_t)n_cu * 8 + n_jobs - 1) / n_jobs;
  if (cap < 1) cap = 1;
  const uint32_t blocks = (uint32_t)(blocks_needed < cap ? blocks_needed : cap);
  if (one) hipLaunchKernelGGL((mx_one<FMT, KIND, LT>), dim3(blocks), dim3(kBlockThreads), 0, s, *one);
  else
    for (uint32_t first = 0; first < n_jobs; first += kMaxGridRows) {  // gridDim.y holds at most 65,535 rows
      const uint32_t rows = n_jobs - first < kMaxGridRows ? n_jobs - first : kMaxGridRows;
      hipLaunchKernelGGL((mx_batch<FMT, KIND, LT>), dim3(blocks, rows), dim3(kBlockThreads), 0, s, jobs + first);
    }
  return hipGetLastError();
}

template <int FMT>
hipError_t dispatch(Kind kind, dq_dtype dtype, bool has_local, const MxJob *one, const MxJob *jobs, uint32_t n_jobs,
                    uint64_t max_entries, uint32_t n_cu, hipStream_t s) {
  const bool f32 = dtype == DQ_F32;
  switch (kind) {
    case kCompress:
      return f32 ? go<FMT, kCompress, float>(one, jobs, n_jobs, max_entries, n_cu, s)
                 : go<FMT, kCompress, uint16_t>(one, jobs, n_jobs, max_entries, n_cu, s);
    case kDar:
      return f32 ? go<FMT, kDar, float>(one, jobs, n_jobs, max_entries, n_cu, s)
                 : go<FMT, kDar, uint16_t>(one, jobs, n_jobs, max_entries, n_cu, s);
    default:
      if (!has_local) return go<FMT, kDecompress, NoLocal>(one, jobs, n_jobs, max_entries, n_cu, s);
      return f32 ? go<FMT, kDecompress, float>(one, jobs, n_jobs, max_entries, n_cu, s)
                 : go<FMT, kDecompress, uint16_t>(one, jobs, n_jobs, max_entries, n_cu, s);
  }
}

hipError_t dispatch_fmt(Kind kind, dq_codec fmt, dq_dtype dtype, bool has_local, const MxJob *one, const MxJob *jobs,
                        uint32_t n_jobs, uint64_t max_entries, uint32_t n_cu, hipStream_t s) {
  switch (fmt) {
    case DQ_MXFP8_E4M3: return dispatch<DQ_MXFP8_E4M3>(kind, dtype, has_local, one, jobs, n_jobs, max_entries, n_cu, s);
    case DQ_MXFP6_E3M2: return dispatch<DQ_MXFP6_E3M2>(kind, dtype, has_local, one, jobs, n_jobs, max_entries, n_cu, s);
    case DQ_MXFP4_E2M1: return dispatch<DQ_MXFP4_E2M1>(kind, dtype, has_local, one, jobs, n_jobs, max_entries, n_cu, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

hipError_t mx_launch_one(Kind kind, dq_codec fmt, dq_dtype dtype, bool has_local, const MxJob &job, uint32_t n_cu,
                         hipStream_t s) {
  return dispatch_fmt(kind, fmt, dtype, has_local, &job, nullptr, 1, job.n_entries, n_cu, s);
}
hipError_t mx_launch_batch(Kind kind, dq_codec fmt, dq_dtype dtype, bool has_local, const MxJob *jobs, uint32_t n_jobs,
                           uint64_t max_entries, uint32_t n_cu, hipStream_t s) {
  return dispatch_fmt(kind, fmt, dtype, has_local, nullptr, jobs, n_jobs, max_entries, n_cu, s);
}

}  // namespace dq

// ---- C ABI ----------------------------------------------------------------------------
namespace {
bool al16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool is_mx_fmt(dq_codec f) { return f == DQ_MXFP8_E4M3 || f == DQ_MXFP6_E3M2 || f == DQ_MXFP4_E2M1; }
int code_bits(dq_codec f) { return f == DQ_MXFP8_E4M3 ? 8 : f == DQ_MXFP6_E3M2 ? 6 : 4; }
uint32_t device_cus() {
  static thread_local int cached = 0;
  if (!cached) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      cached = prop.multiProcessorCount;
    else
      cached = 256;
  }
  return (uint32_t)cached;
}
}  // namespace

extern "C" {

size_t dq_mx_packed_bytes(dq_codec fmt, uint64_t n_entries) {
  if (!is_mx_fmt(fmt) || n_entries % 256) return 0;
  const uint64_t blocks = n_entries / 32;
  const uint64_t sz = blocks * (uint64_t)(code_bits(fmt) * 4) + blocks;
  return (size_t)((sz + 15) & ~(uint64_t)15);
}

dq_status dq_mx_compress(dq_codec fmt, const void *local, dq_dtype dtype, uint64_t n_entries, void *packed_out,
                         void *hip_stream) {
  if (!is_mx_fmt(fmt) || !local || !packed_out || n_entries % 256 || (dtype != DQ_F32 && dtype != DQ_BF16))
    return DQ_EINVAL;
  if (!al16(local) || !al16(packed_out)) return DQ_EALIGN;
  dq::MxJob j{nullptr, local, packed_out, n_entries};
  return dq::hip_status(dq::mx_launch_one(dq::kCompress, fmt, dtype, true, j, device_cus(), (hipStream_t)hip_stream));
}

dq_status dq_mx_dar_hop(dq_codec fmt, const void *packed_in, const void *local, dq_dtype dtype, uint64_t n_entries,
                        void *packed_out, void *hip_stream) {
  if (!is_mx_fmt(fmt) || !packed_in || !local || !packed_out || n_entries % 256 ||
      (dtype != DQ_F32 && dtype != DQ_BF16))
    return DQ_EINVAL;
  if (!al16(packed_in) || !al16(local) || !al16(packed_out)) return DQ_EALIGN;
  dq::MxJob j{(const uint8_t *)packed_in, local, packed_out, n_entries};
  return dq::hip_status(dq::mx_launch_one(dq::kDar, fmt, dtype, true, j, device_cus(), (hipStream_t)hip_stream));
}

dq_status dq_mx_decompress(dq_codec fmt, const void *packed_in, const void *local_or_null, dq_dtype dtype,
                           uint64_t n_entries, float *out, void *hip_stream) {
  if (!is_mx_fmt(fmt) || !packed_in || !out || n_entries % 256) return DQ_EINVAL;
  if (local_or_null && dtype != DQ_F32 && dtype != DQ_BF16) return DQ_EINVAL;
  if (!al16(packed_in) || !al16(out) || !al16(local_or_null)) return DQ_EALIGN;
  dq::MxJob j{(const uint8_t *)packed_in, local_or_null, out, n_entries};
  return dq::hip_status(dq::mx_launch_one(dq::kDecompress, fmt, dtype, local_or_null != nullptr, j, device_cus(),
                           (hipStream_t)hip_stream));
}

}  // extern "C"
