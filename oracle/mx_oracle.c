/*
 * mx_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain CPU implementation of the OCP Microscaling (MX) comparison codec in the
 * hop loop of a compressed reduce-scatter: blocks of 32 values share a power-of-two
 * scale stored as one E8M0 byte, elements are FP8 E4M3, FP6 E3M2 or FP4 E2M1 --
 * the three formats the paper compares against (Section 5, "Baseline compression
 * schemes").  The conversion follows the OCP MX v1.0 specification that the paper
 * cites: shared exponent = floor(log2(max|v|)) - emax_elem, elements = v / 2^shared
 * rounded to nearest, ties to even, and clamped to the largest normal (the formats
 * have no infinity to overflow into).  Nothing here is shared with the GPU library.
 *
 * fmt: 1 = E4M3 (bias 7, 3 mantissa bits, max 448), 2 = E3M2 (bias 3, 2 mantissa
 * bits, max 28), 3 = E2M1 (bias 1, 1 mantissa bit, max 6).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int ebits, mbits, bias, emax; /* emax: exponent of the largest normal */
  float max_normal;
  int code_bits;
} mx_format;

static const mx_format MXF[4] = {
    {0, 0, 0, 0, 0.0f, 0},
    {4, 3, 7, 8, 448.0f, 8},
    {3, 2, 3, 4, 28.0f, 6},
    {2, 1, 1, 2, 6.0f, 4},
};

static float mx_bf16(uint16_t h) {
  uint32_t b = (uint32_t)h << 16;
  float f;
  memcpy(&f, &b, 4);
  return f;
}

/* E8M0 byte for a block whose largest magnitude is m: floor(log2 m) - emax + 127,
 * clamped to [0, 254]; 0 for an all-zero block (255 would mean NaN and is never
 * produced). */
int mxo_block_scale(int fmt, float m) {
  if (!(m > 0.0f)) return 0;
  int ex;
  (void)frexpf(m, &ex); /* m = f * 2^ex, f in [0.5, 1)  ->  floor(log2 m) = ex - 1 */
  int e = (ex - 1) - MXF[fmt].emax + 127;
  if (e < 0) e = 0;
  if (e > 254) e = 254;
  return e;
}

/* Element code of v under the block scale 2^(e-127): sign bit on top, then the
 * exponent field, then the mantissa. */
uint32_t mxo_encode_elem(int fmt, float v, int e) {
  const mx_format *F = &MXF[fmt];
  uint32_t sign = signbit(v) ? 1u : 0u;
  float a = ldexpf(fabsf(v), 127 - e); /* exact power-of-two scaling */
  if (a >= F->max_normal) a = F->max_normal;
  uint32_t field = 0, mant = 0;
  if (a > 0.0f) {
    int ex;
    (void)frexpf(a, &ex);
    int E = ex - 1;                     /* floor(log2 a) */
    int emin = 1 - F->bias;             /* exponent of the smallest normal */
    if (E < emin) E = emin;             /* subnormal range: fixed quantum */
    float quantum = ldexpf(1.0f, E - F->mbits);
    float q = rintf(a / quantum);       /* nearest, ties to even; the division is exact */
    float val = q * quantum;
    if (val > F->max_normal) val = F->max_normal;
    if (val > 0.0f) {
      (void)frexpf(val, &ex);
      int E2 = ex - 1;
      if (E2 < emin) { /* subnormal: field 0, mantissa counts quanta */
        field = 0;
        mant = (uint32_t)(val / ldexpf(1.0f, emin - F->mbits));
      } else {
        field = (uint32_t)(E2 + F->bias);
        mant = (uint32_t)(val / ldexpf(1.0f, E2 - F->mbits)) - (1u << F->mbits);
      }
    }
  }
  return (sign << (F->ebits + F->mbits)) | (field << F->mbits) | mant;
}

/* Value of an element code times the block scale 2^(e-127). */
float mxo_decode_elem(int fmt, uint32_t code, int e) {
  const mx_format *F = &MXF[fmt];
  uint32_t mant = code & ((1u << F->mbits) - 1u);
  uint32_t field = (code >> F->mbits) & ((1u << F->ebits) - 1u);
  uint32_t sign = (code >> (F->ebits + F->mbits)) & 1u;
  float val;
  if (field == 0) val = ldexpf((float)mant, 1 - F->bias - F->mbits);
  else val = ldexpf((float)(mant + (1u << F->mbits)), (int)field - F->bias - F->mbits);
  val = ldexpf(val, e - 127);
  return sign ? -val : val;
}

/* Packed layout: [element codes, code_bits*4 bytes per block of 32][one E8M0 byte per
 * block], each array 16-byte aligned (n_entries is a multiple of 256), total rounded
 * up to 16.  Element k of a block sits at bit offset k*code_bits of the block's code
 * bytes, little-endian. */
uint64_t mxo_packed_bytes(int fmt, uint64_t n_entries) {
  uint64_t blocks = n_entries / 32;
  uint64_t sz = blocks * (uint64_t)(MXF[fmt].code_bits * 4) + blocks;
  return (sz + 15ull) & ~15ull;
}

static float mx_local(const void *local, int dtype, uint64_t j) {
  return dtype == 0 ? ((const float *)local)[j] : mx_bf16(((const uint16_t *)local)[j]);
}

static void mx_put(uint8_t *blk, int cb, int k, uint32_t code) {
  int bit = k * cb;
  for (int i = 0; i < cb; ++i, ++bit)
    if ((code >> i) & 1u) blk[bit >> 3] |= (uint8_t)(1u << (bit & 7));
}
static uint32_t mx_get(const uint8_t *blk, int cb, int k) {
  int bit = k * cb;
  uint32_t code = 0;
  for (int i = 0; i < cb; ++i, ++bit) code |= (uint32_t)((blk[bit >> 3] >> (bit & 7)) & 1u) << i;
  return code;
}

static void mx_encode_block(int fmt, const float v[32], uint8_t *blk, uint8_t *scale) {
  int cb = MXF[fmt].code_bits;
  float m = 0.0f;
  for (int k = 0; k < 32; ++k) m = fmaxf(m, fabsf(v[k]));
  int e = mxo_block_scale(fmt, m);
  *scale = (uint8_t)e;
  memset(blk, 0, (size_t)(cb * 4));
  for (int k = 0; k < 32; ++k) mx_put(blk, cb, k, mxo_encode_elem(fmt, v[k], e));
}

void mxo_compress(int fmt, uint64_t n, const void *local, int dtype, void *packed_out) {
  int cb = MXF[fmt].code_bits;
  uint8_t *codes = (uint8_t *)packed_out, *scales = codes + (n / 32) * (uint64_t)(cb * 4);
  memset(packed_out, 0, mxo_packed_bytes(fmt, n));
  for (uint64_t b = 0; b < n / 32; ++b) {
    float v[32];
    for (int k = 0; k < 32; ++k) v[k] = mx_local(local, dtype, b * 32 + k);
    mx_encode_block(fmt, v, codes + b * (uint64_t)(cb * 4), scales + b);
  }
}

/* decode the partial sum, add the local slice (one fused multiply-add per entry:
 * element value times the power-of-two scale plus local), re-encode */
void mxo_dar_hop(int fmt, uint64_t n, const void *packed_in, const void *local, int dtype, void *packed_out) {
  int cb = MXF[fmt].code_bits;
  uint64_t bytes = mxo_packed_bytes(fmt, n);
  uint8_t *tmp = (uint8_t *)calloc(1, bytes);
  const uint8_t *ic = (const uint8_t *)packed_in, *is = ic + (n / 32) * (uint64_t)(cb * 4);
  uint8_t *oc = tmp, *os = tmp + (n / 32) * (uint64_t)(cb * 4);
  for (uint64_t b = 0; b < n / 32; ++b) {
    float v[32];
    int e = is[b];
    float X = ldexpf(1.0f, e - 127);
    for (int k = 0; k < 32; ++k) {
      float el = mxo_decode_elem(fmt, mx_get(ic + b * (uint64_t)(cb * 4), cb, k), 127); /* unscaled element */
      v[k] = fmaf(el, X, mx_local(local, dtype, b * 32 + k));
    }
    mx_encode_block(fmt, v, oc + b * (uint64_t)(cb * 4), os + b);
  }
  memcpy(packed_out, tmp, bytes);
  free(tmp);
}

void mxo_decompress(int fmt, uint64_t n, const void *packed_in, const void *local_or_null, int dtype, float *out) {
  int cb = MXF[fmt].code_bits;
  const uint8_t *ic = (const uint8_t *)packed_in, *is = ic + (n / 32) * (uint64_t)(cb * 4);
  for (uint64_t b = 0; b < n / 32; ++b) {
    int e = is[b];
    float X = ldexpf(1.0f, e - 127);
    for (int k = 0; k < 32; ++k) {
      float el = mxo_decode_elem(fmt, mx_get(ic + b * (uint64_t)(cb * 4), cb, k), 127);
      out[b * 32 + k] = local_or_null ? fmaf(el, X, mx_local(local_or_null, dtype, b * 32 + k)) : el * X;
    }
  }
}
