/*
 * dq_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-threaded CPU implementation of what DynamiQ's
 * compressed-all-reduce hot path computes: first-hop compress, the fused
 * decompress-accumulate-recompress (DAR) hop, and decompress(+accumulate),
 * for the grouped non-uniform stochastic quantizer of the paper's Section 3.3
 * with hierarchical scales and correlated rounding.  It exists only so that
 * tests, the smoke check and the benchmark's cpu_baseline leg can compare the
 * HIP kernels against it.  It shares no code, table, header or constant
 * generator with the GPU library and never calls it.
 *
 * Everything below takes the algorithm's steps in the paper's order:
 *   - stochastic quantization onto a level set          (Section 2.1)
 *   - groups of s=16 and super-groups of S=256 entries  (Sections 2.2, 5 "configuration")
 *   - level set Q = { f(eps, r) }                        (Section 3.3, "Non-uniform quantization")
 *   - normalisation by the group maximum, separate sign  (Section 3.3)
 *   - u8 group scale r_G, bf16 super-group scale sf_SG   (Section 3.3, "Hierarchical quantization")
 *   - u_i = (pi_i + gamma_i) / n                         (Section 3.3, "Correlated rounding")
 *   - who runs which kernel on a hop                     (Section 3.4, "Fused kernels"; Section 4)
 * Where the paper is silent (arithmetic order, rounding of the scales, the
 * random stream layout, the wire format) the choices made are spelled out in
 * the comments of each function; they are all IEEE-754 binary32 operations,
 * one rounding per written operation, with fmaf() where a fused multiply-add
 * is meant.  Build with -ffp-contract=off so the compiler fuses nothing else.
 *
 * Random numbers are inputs to the *_core functions (bytes and the permuted
 * slot), so tests can enumerate every outcome; the *_sg wrappers draw them from
 * a counter-based Philox4x32-10 generator.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define DQO_GROUP 16
#define DQO_SG 256
#define DQO_GROUPS_PER_SG 16

typedef struct {
  double g4, g8;      /* 1 + 2*eps^2 for the 4-bit and 8-bit level sets */
  uint64_t seed;      /* shared PRNG seed (Section 2.4: workers share a seed) */
  uint32_t round;     /* training round, so that every round draws fresh numbers */
  uint32_t n_workers; /* n in u_i = (pi_i + gamma_i)/n */
  uint32_t independent; /* 1: every worker rounds on its own, u = gamma (the baseline that Section 2.4 improves on) */
  uint32_t reserved;
} dqo_config;

typedef struct {
  dqo_config cfg;
  /* wi = 0,1,2 <-> b = 2,4,8 bits; R = 2^(b-1)-1 = 1,7,127 */
  float T[3][128]; /* levels, T[wi][0..R] */
  float D[3][128]; /* gaps   D[wi][r] = T[r+1]-T[r], r < R */
  float inv_n, s_n;
} dqo_ctx;

static const int DQO_BITS[3] = {2, 4, 8};
static const int DQO_R[3] = {1, 7, 127};

static float bits_to_f32(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
static uint32_t f32_to_bits(float f) { uint32_t b; memcpy(&b, &f, 4); return b; }
static float bf16_to_f32(uint16_t h) { return bits_to_f32((uint32_t)h << 16); }

/* ---------------------------------------------------------------- levels */

/* Section 3.3: f(eps, r) = ((1+2eps^2)^r - 1) / ((1+2eps^2)^(2^(b-1)-1) - 1),
 * r = 0 .. 2^(b-1)-1.  g = 1+2eps^2 is the parameter (the paper never prints
 * eps).  Powers by repeated multiplication in double so that any language
 * yields the same table; the ends are forced to 0 and 1.  For b = 2 the set is
 * {0, 1} whatever g is.  Returns 0 on success, -1 if the fp32 levels are not
 * strictly increasing (g too close to 1 or too large). */
int dqo_levels(int wi, double g, float *T, float *D) {
  int R = DQO_R[wi];
  double pw[128];
  pw[0] = 1.0;
  for (int r = 1; r <= R; ++r) pw[r] = pw[r - 1] * g;
  double den = pw[R] - 1.0;
  for (int r = 0; r <= R; ++r) T[r] = (R == 1) ? (float)r : (float)((pw[r] - 1.0) / den);
  T[0] = 0.0f;
  T[R] = 1.0f;
  for (int r = 0; r < R; ++r) {
    D[r] = T[r + 1] - T[r];
    if (!(D[r] > 0.0f)) return -1;
  }
  return 0;
}

dqo_ctx *dqo_create(const dqo_config *cfg) {
  if (cfg->n_workers < 1 || cfg->n_workers > 8192) return NULL;
  dqo_ctx *c = (dqo_ctx *)calloc(1, sizeof(dqo_ctx));
  c->cfg = *cfg;
  if (dqo_levels(0, 2.0, c->T[0], c->D[0]) || dqo_levels(1, cfg->g4, c->T[1], c->D[1]) ||
      dqo_levels(2, cfg->g8, c->T[2], c->D[2])) {
    free(c);
    return NULL;
  }
  /* constants of the entry uniform (see dqo_entry_uniform) */
  /* independent rounding is the case n = 1 of the same formula: one interval, u = (byte + 1/2)/256 */
  c->inv_n = cfg->independent ? 1.0f : 1.0f / (float)cfg->n_workers;
  c->s_n = c->inv_n * (1.0f / 256.0f);
  return c;
}
void dqo_destroy(dqo_ctx *c) { free(c); }
const float *dqo_table_T(const dqo_ctx *c, int wi) { return c->T[wi]; }
const float *dqo_table_D(const dqo_ctx *c, int wi) { return c->D[wi]; }

/* ---------------------------------------------------------------- Philox */

/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random
 * numbers: as easy as 1, 2, 3", SC'11).  One round: two 32x32->64 products of
 * counter words 0 and 2 with the two multipliers; the high halves are xored
 * with the other counter words and the round key; the key is bumped by the
 * Weyl constants between rounds. */
void dqo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int i = 0; i < 10; ++i) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

enum { DQO_STREAM_GAMMA = 0, DQO_STREAM_SCALE = 1, DQO_STREAM_PERM = 2 };

static void dqo_draw(const dqo_ctx *c, uint64_t index, uint32_t stream, uint32_t rank16, uint32_t out[4]) {
  uint32_t ctr[4] = {(uint32_t)index, (uint32_t)(index >> 32), c->cfg.round, (stream << 16) | (rank16 & 0xFFFFu)};
  uint32_t key[2] = {(uint32_t)c->cfg.seed, (uint32_t)(c->cfg.seed >> 32)};
  dqo_philox4x32_10(ctr, key, out);
}
static uint8_t word_byte(const uint32_t w[4], int k) { return (uint8_t)(w[k >> 2] >> (8 * (k & 3))); }

/* The random numbers one worker needs to compress super-group `sg` (its global,
 * post-reorder index), per Section 3.3 "Correlated rounding":
 *   gamma[256]  one byte per entry:   stream GAMMA, counter = global group index 16*sg+g,
 *               private to the worker (rank in the counter); entry k of the group
 *               takes byte k of the 16 output bytes (little-endian in words 0..3).
 *   scale_byte[16] one byte per group: stream SCALE, counter = sg, private to the worker
 *               (the scale rounding must be independent of the entry rounding, Section 3.3).
 *   slot        pi_rank for the super-group's first group: stream PERM, counter = sg,
 *               NOT keyed by the worker, so all workers derive the same random permutation
 *               of 0..n-1 without communicating (dqo_perm_slot below); group g of the
 *               super-group uses (slot + g) mod n, so that a worker's 16 groups are spread
 *               over the n intervals. */

/* The shared random permutation pi of 0..n-1 (Section 3.3), evaluated at one worker index
 * without building the permutation.  With k = ceil(log2 n) and the four words w0..w3 of the
 * PERM draw, three rounds of
 *     y <- reverse_k( ((w_t | 1) * y + (w_t >> 16)) mod 2^k )          t = 0, 1, 2
 * map the k-bit integers one-to-one onto themselves: multiplying by an odd number and adding
 * a constant are bijections mod 2^k (they carry information from low bits to high bits), and
 * reversing the order of the k bits is a bijection that swaps the two directions.  For n
 * below 2^k the walk is repeated until it lands below n ("cycle walking": following a
 * permutation of 0..2^k-1 from a point below n until it returns below n is a permutation of
 * 0..n-1).  A final rotation by floor(w3 * n / 2^32) makes every worker's slot uniform on
 * 0..n-1 whatever the rounds do.  The multipliers use bits 0..12 of a word and the added
 * constants bits 16..28 (n <= 8192, so k <= 13): independent bits. */
static uint32_t reverse_bits(uint32_t y, uint32_t k) {
  uint32_t r = 0;
  for (uint32_t i = 0; i < k; ++i) r |= ((y >> i) & 1u) << (k - 1 - i);
  return r;
}
uint32_t dqo_perm_bits(uint32_t n) {
  uint32_t k = 0;
  while ((1u << k) < n) ++k;
  return k;
}
static uint32_t perm_rounds(const uint32_t w[4], uint32_t k, uint32_t y) {
  const uint32_t mask = (1u << k) - 1u;
  for (int t = 0; t < 3; ++t) y = reverse_bits(((w[t] | 1u) * y + (w[t] >> 16)) & mask, k);
  return y;
}
uint32_t dqo_perm_slot(const uint32_t w[4], uint32_t n, uint32_t rank) {
  const uint32_t k = dqo_perm_bits(n);
  uint32_t y = perm_rounds(w, k, rank);
  while (y >= n) y = perm_rounds(w, k, y);
  const uint32_t rot = (uint32_t)(((uint64_t)w[3] * n) >> 32);
  return (y + rot) % n;
}

void dqo_draw_sg(const dqo_ctx *c, uint64_t sg, uint32_t rank, uint8_t gamma[DQO_SG],
                 uint8_t scale_byte[DQO_GROUPS_PER_SG], uint32_t *slot) {
  uint32_t w[4];
  for (int g = 0; g < DQO_GROUPS_PER_SG; ++g) {
    dqo_draw(c, sg * 16 + (uint64_t)g, DQO_STREAM_GAMMA, rank, w);
    for (int k = 0; k < DQO_GROUP; ++k) gamma[g * DQO_GROUP + k] = word_byte(w, k);
  }
  dqo_draw(c, sg, DQO_STREAM_SCALE, rank, w);
  for (int g = 0; g < DQO_GROUPS_PER_SG; ++g) scale_byte[g] = word_byte(w, g);
  dqo_draw(c, sg, DQO_STREAM_PERM, 0xFFFFu, w);
  *slot = c->cfg.independent ? 0u : dqo_perm_slot(w, c->cfg.n_workers, rank);
}

/* ---------------------------------------------------------------- quantizer pieces */

/* u_i = (pi_i + gamma_i)/n with gamma_i = (byte + 1/2)/256, evaluated as
 *   inv_n = 1/n;  s_n = inv_n/256;  o = (pi_i + 1/512) * inv_n;  u = fma(byte, s_n, o).
 * For n a power of two every step is exact. */
float dqo_entry_uniform(const dqo_ctx *c, uint32_t slot, uint8_t byte) {
  float o = ((float)slot + (1.0f / 512.0f)) * c->inv_n;
  return fmaf((float)byte, c->s_n, o);
}

/* Section 2.1: x_dn = max{q in Q : q <= x}, x_up the next level; round up with
 * probability (x - x_dn)/(x_up - x_dn).  With a uniform u the event "u < p" is
 * written division-free as  T[r] + u*D[r] < x  (one fma, one compare).
 * Returns the level index. */
int dqo_sq_index(const float *T, const float *D, int R, float x, float u) {
  int r = 0;
  while (r < R && T[r + 1] <= x) ++r; /* r = max{ r : T[r] <= x } */
  if (r == R) return R;
  return r + (fmaf(u, D[r], T[r]) < x ? 1 : 0);
}

/* Smallest bf16 that is >= m (m >= 0, finite): the super-group scale is stored
 * in 16 bits (Section 5, "per-super-group scaling parameters are kept as BF16");
 * rounding up keeps max|G|/sf_SG <= 1 so that r_G never exceeds 255. */
uint16_t dqo_bf16_ceil(float m) {
  uint32_t b = f32_to_bits(m);
  uint32_t h = b >> 16;
  if (b & 0xFFFFu) h += 1;
  return (uint16_t)h;
}

/* Super-groups whose largest magnitude is below 2^-100 are encoded as all-zero:
 * their reciprocals would overflow binary32. */
#define DQO_SF_MIN_BITS 0x0D80u /* bf16 pattern of 2^-100 */

/* Encode one super-group of 256 values v[] at width index wi.
 * Random inputs: gamma[256], scale_byte[16], slot = pi_rank of group 0 (group g
 * uses (slot + g) mod n).
 * Outputs: code[256] = (sign << (b-1)) | r, rG[16], *sf_bits (bf16 pattern). */
void dqo_encode_sg_core(const dqo_ctx *c, int wi, const float v[DQO_SG], const uint8_t gamma[DQO_SG],
                        const uint8_t scale_byte[DQO_GROUPS_PER_SG], uint32_t slot, uint8_t code[DQO_SG],
                        uint8_t rG[DQO_GROUPS_PER_SG], uint16_t *sf_bits) {
  const int b = DQO_BITS[wi], R = DQO_R[wi];
  const float *T = c->T[wi], *D = c->D[wi];
  /* sf_SG = max |SG|, kept in bf16 (rounded up) */
  float M = 0.0f;
  for (int k = 0; k < DQO_SG; ++k) M = fmaxf(M, fabsf(v[k]));
  uint16_t sfb = dqo_bf16_ceil(M);
  if (sfb < DQO_SF_MIN_BITS) sfb = 0;
  *sf_bits = sfb;
  float sf = bf16_to_f32(sfb);
  float cs = (sfb != 0) ? 255.0f / sf : 0.0f; /* one divide per super-group */
  for (int g = 0; g < DQO_GROUPS_PER_SG; ++g) {
    const float *vg = v + g * DQO_GROUP;
    uint8_t *cg = code + g * DQO_GROUP;
    float m = 0.0f;
    for (int k = 0; k < DQO_GROUP; ++k) m = fmaxf(m, fabsf(vg[k]));
    /* group scale: uniform stochastic quantization of max|G| onto {r*sf_SG/255},
     * so that E[sf_G] = max|G| */
    int rg = 0;
    if (sfb != 0) {
      float t = fminf(m * cs, 255.0f);
      float fl = floorf(t);
      float us = ((float)scale_byte[g] + 0.5f) * (1.0f / 256.0f);
      rg = (int)fl + (us < t - fl ? 1 : 0);
    }
    rG[g] = (uint8_t)rg;
    if (rg == 0) { /* the group decodes to zero whatever its codes are: keep signs, r = 0 */
      for (int k = 0; k < DQO_GROUP; ++k) cg[k] = (uint8_t)((f32_to_bits(vg[k]) >> 31) << (b - 1));
      continue;
    }
    /* entries: normalise by the true group maximum, stochastic-quantize onto Q */
    float inv = 1.0f / m; /* one divide per group */
    for (int k = 0; k < DQO_GROUP; ++k) {
      float x = fminf(fabsf(vg[k]) * inv, 1.0f);
      const uint32_t pi = c->cfg.independent ? 0u : (slot + (uint32_t)g) % c->cfg.n_workers;
      float u = dqo_entry_uniform(c, pi, gamma[g * DQO_GROUP + k]);
      int r = dqo_sq_index(T, D, R, x, u);
      cg[k] = (uint8_t)(((f32_to_bits(vg[k]) >> 31) << (b - 1)) | (uint32_t)r);
    }
  }
}

/* Decode one super-group: estimate = sign * f(eps, r) * sf_G with
 * sf_G = r_G * (sf_SG/255)  (Section 3.3).  With a local slice the estimate is
 * accumulated by one fused multiply-add, out = fma(sign*T[r], sf_G, local);
 * without, out = sign*T[r] * sf_G. */
void dqo_decode_sg_core(const dqo_ctx *c, int wi, const uint8_t code[DQO_SG], const uint8_t rG[DQO_GROUPS_PER_SG],
                        uint16_t sf_bits, const float *local_or_null, float out[DQO_SG]) {
  const int b = DQO_BITS[wi], R = DQO_R[wi];
  const float *T = c->T[wi];
  float step = bf16_to_f32(sf_bits) / 255.0f; /* one divide per super-group */
  for (int g = 0; g < DQO_GROUPS_PER_SG; ++g) {
    float sfg = (float)rG[g] * step;
    for (int k = 0; k < DQO_GROUP; ++k) {
      int i = g * DQO_GROUP + k;
      uint32_t cd = code[i];
      float t = T[cd & (uint32_t)R];
      if ((cd >> (b - 1)) & 1u) t = -t;
      out[i] = local_or_null ? fmaf(t, sfg, local_or_null[i]) : t * sfg;
    }
  }
}

/* ---------------------------------------------------------------- wire format */

/* A chunk is a run of super-groups with global indices first_sg, first_sg+1, ...;
 * the first n_sg[0] use 2 bits, the next n_sg[1] 4 bits, then n_sg[2] at 8 bits and
 * the last n_sg[3] at 16 bits (super-groups are reordered by increasing width,
 * Section 3.5; "16 bits corresponds to uncompressed values", Section 3.2: such a
 * super-group travels as 256 raw bf16 numbers, without scales).  Packed buffer,
 * structure of arrays, every array 16-byte aligned, each in super-group order:
 *   [2-bit codes: 64 B per SG][4-bit codes: 128 B per SG][8-bit codes: 256 B per SG]
 *   [16-bit values: 512 B per SG]
 *   [group scales: 16 u8 per coded SG][super-group scales: one u16 (bf16 pattern) per coded SG]
 * where the coded super-groups are those at 2, 4 and 8 bits.  Entry k of a coded
 * super-group sits at bit offset k*b of its code block, little-endian.
 * The total is rounded up to a multiple of 16. */
typedef struct {
  uint64_t first_sg;
  uint32_t n_sg[4];
} dqo_chunk;

static uint64_t chunk_coded_sg(const dqo_chunk *ch) { return (uint64_t)ch->n_sg[0] + ch->n_sg[1] + ch->n_sg[2]; }
static uint64_t chunk_total_sg(const dqo_chunk *ch) { return chunk_coded_sg(ch) + ch->n_sg[3]; }
static const uint64_t DQO_CODE_BYTES[4] = {64, 128, 256, 512};

uint64_t dqo_packed_bytes(const dqo_chunk *ch) {
  uint64_t n = chunk_coded_sg(ch);
  uint64_t sz = 64ull * ch->n_sg[0] + 128ull * ch->n_sg[1] + 256ull * ch->n_sg[2] + 512ull * ch->n_sg[3] + 16ull * n + 2ull * n;
  return (sz + 15ull) & ~15ull;
}

typedef struct {
  uint8_t *codes[4];
  uint8_t *gscale;
  uint8_t *sgscale;
} dqo_view;

static dqo_view chunk_view(const dqo_chunk *ch, void *packed) {
  dqo_view v;
  uint8_t *p = (uint8_t *)packed;
  v.codes[0] = p;
  v.codes[1] = v.codes[0] + 64ull * ch->n_sg[0];
  v.codes[2] = v.codes[1] + 128ull * ch->n_sg[1];
  v.codes[3] = v.codes[2] + 256ull * ch->n_sg[2];
  v.gscale = v.codes[3] + 512ull * ch->n_sg[3];
  v.sgscale = v.gscale + 16ull * chunk_coded_sg(ch);
  return v;
}

/* fp32 -> bf16, round to nearest, ties to even (finite values) */
static uint16_t f32_to_bf16_rne(float f) {
  uint32_t b = f32_to_bits(f);
  uint32_t keep = b >> 16, rest = b & 0xFFFFu;
  if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
  return (uint16_t)keep;
}

static void pack_codes(int b, const uint8_t code[DQO_SG], uint8_t *dst) {
  memset(dst, 0, (size_t)(DQO_SG * b / 8));
  for (int k = 0; k < DQO_SG; ++k) {
    int bit = k * b;
    dst[bit >> 3] |= (uint8_t)(code[k] << (bit & 7));
  }
}
static void unpack_codes(int b, const uint8_t *src, uint8_t code[DQO_SG]) {
  for (int k = 0; k < DQO_SG; ++k) {
    int bit = k * b;
    code[k] = (uint8_t)((src[bit >> 3] >> (bit & 7)) & ((1u << b) - 1u));
  }
}

/* local slice element j as fp32; dtype 0 = fp32, 1 = bf16 (exact widening) */
static float local_at(const void *local, int dtype, uint64_t j) {
  if (dtype == 0) return ((const float *)local)[j];
  return bf16_to_f32(((const uint16_t *)local)[j]);
}

/* Section 3.1: every worker subtracts the super-group's mean mu_j from its entries before
 * they are quantized.  Reading: the subtraction is one fp32 operation on the widened entry,
 * done where the entry enters the main stage (never stored back in the gradient's dtype:
 * rounding x - mu to bf16 returns x whenever |mu| is below half an ulp of x, and then all
 * n workers err by +mu together).  mu is indexed by the super-group's place in the chunk;
 * NULL = nothing is subtracted. */
static void local_sg(const void *local, int dtype, const float *mu_or_null, uint64_t j, float v[DQO_SG]) {
  for (int k = 0; k < DQO_SG; ++k) {
    const float x = local_at(local, dtype, j * DQO_SG + k);
    v[k] = mu_or_null ? x - mu_or_null[j] : x;
  }
}

/* width index and position inside its code array of the j-th super-group of a chunk */
static int sg_width(const dqo_chunk *ch, uint64_t j, uint64_t *pos) {
  if (j < ch->n_sg[0]) { *pos = j; return 0; }
  j -= ch->n_sg[0];
  if (j < ch->n_sg[1]) { *pos = j; return 1; }
  j -= ch->n_sg[1];
  if (j < ch->n_sg[2]) { *pos = j; return 2; }
  *pos = j - ch->n_sg[2];
  return 3;
}

/* ---------------------------------------------------------------- the three kernels */

/* Leaf node: compress the local chunk (Section 4, kernel 1).  `rank` is the
 * worker doing the compression. */
void dqo_compress(const dqo_ctx *c, const dqo_chunk *ch, uint32_t rank, const void *local, int dtype,
                  const float *mu_or_null, void *packed_out) {
  dqo_view o = chunk_view(ch, packed_out);
  uint64_t n = chunk_total_sg(ch);
  memset(packed_out, 0, dqo_packed_bytes(ch));
  for (uint64_t j = 0; j < n; ++j) {
    uint64_t pos;
    int wi = sg_width(ch, j, &pos);
    float v[DQO_SG];
    uint8_t gamma[DQO_SG], sb[16], code[DQO_SG], rG[16];
    uint16_t sf;
    uint32_t slot;
    local_sg(local, dtype, mu_or_null, j, v);
    if (wi == 3) { /* uncompressed: the values themselves, as bf16 */
      uint16_t *raw = (uint16_t *)(o.codes[3] + pos * 512);
      for (int k = 0; k < DQO_SG; ++k) raw[k] = f32_to_bf16_rne(v[k]);
      continue;
    }
    dqo_draw_sg(c, ch->first_sg + j, rank, gamma, sb, &slot);
    dqo_encode_sg_core(c, wi, v, gamma, sb, slot, code, rG, &sf);
    pack_codes(DQO_BITS[wi], code, o.codes[wi] + pos * DQO_CODE_BYTES[wi]);
    memcpy(o.gscale + 16 * j, rG, 16);
    memcpy(o.sgscale + 2 * j, &sf, 2);
  }
}

/* Internal node: decode the received partial sum, add the local slice, re-encode
 * (Section 4, kernel 3); nothing but registers between the three steps. */
void dqo_dar_hop(const dqo_ctx *c, const dqo_chunk *ch, uint32_t rank, const void *packed_in, const void *local,
                 int dtype, const float *mu_or_null, void *packed_out) {
  dqo_view in = chunk_view(ch, (void *)packed_in);
  uint64_t n = chunk_total_sg(ch);
  uint64_t bytes = dqo_packed_bytes(ch);
  uint8_t *tmp = (uint8_t *)calloc(1, bytes); /* packed_out may alias packed_in */
  dqo_view o = chunk_view(ch, tmp);
  for (uint64_t j = 0; j < n; ++j) {
    uint64_t pos;
    int wi = sg_width(ch, j, &pos);
    float loc[DQO_SG], v[DQO_SG];
    uint8_t gamma[DQO_SG], sb[16], code[DQO_SG], rG[16];
    uint16_t sf;
    uint32_t slot;
    local_sg(local, dtype, mu_or_null, j, loc);
    if (wi == 3) { /* uncompressed: bf16 partial sum + local in fp32, rounded back to bf16 */
      const uint16_t *raw_in = (const uint16_t *)(in.codes[3] + pos * 512);
      uint16_t *raw = (uint16_t *)(o.codes[3] + pos * 512);
      for (int k = 0; k < DQO_SG; ++k) raw[k] = f32_to_bf16_rne(bf16_to_f32(raw_in[k]) + loc[k]);
      continue;
    }
    unpack_codes(DQO_BITS[wi], in.codes[wi] + pos * DQO_CODE_BYTES[wi], code);
    memcpy(rG, in.gscale + 16 * j, 16);
    memcpy(&sf, in.sgscale + 2 * j, 2);
    dqo_decode_sg_core(c, wi, code, rG, sf, loc, v);
    dqo_draw_sg(c, ch->first_sg + j, rank, gamma, sb, &slot);
    dqo_encode_sg_core(c, wi, v, gamma, sb, slot, code, rG, &sf);
    pack_codes(DQO_BITS[wi], code, o.codes[wi] + pos * DQO_CODE_BYTES[wi]);
    memcpy(o.gscale + 16 * j, rG, 16);
    memcpy(o.sgscale + 2 * j, &sf, 2);
  }
  memcpy(packed_out, tmp, bytes);
  free(tmp);
}

/* Sink of the reduce-scatter, non-last parents in a butterfly, all-gather
 * receivers: decode, optionally add the local slice (minus its means), write fp32
 * (Section 4, kernels 2 and 4).  out may alias an fp32 local. */
void dqo_decompress(const dqo_ctx *c, const dqo_chunk *ch, const void *packed_in, const void *local_or_null, int dtype,
                    const float *mu_or_null, float *out) {
  dqo_view in = chunk_view(ch, (void *)packed_in);
  uint64_t n = chunk_total_sg(ch);
  for (uint64_t j = 0; j < n; ++j) {
    uint64_t pos;
    int wi = sg_width(ch, j, &pos);
    float loc[DQO_SG], v[DQO_SG];
    uint8_t code[DQO_SG], rG[16];
    uint16_t sf;
    if (local_or_null) local_sg(local_or_null, dtype, mu_or_null, j, loc);
    if (wi == 3) {
      const uint16_t *raw_in = (const uint16_t *)(in.codes[3] + pos * 512);
      for (int k = 0; k < DQO_SG; ++k)
        out[j * DQO_SG + k] = local_or_null ? bf16_to_f32(raw_in[k]) + loc[k] : bf16_to_f32(raw_in[k]);
      continue;
    }
    unpack_codes(DQO_BITS[wi], in.codes[wi] + pos * DQO_CODE_BYTES[wi], code);
    memcpy(rG, in.gscale + 16 * j, 16);
    memcpy(&sf, in.sgscale + 2 * j, 2);
    dqo_decode_sg_core(c, wi, code, rG, sf, local_or_null ? loc : NULL, v);
    memcpy(out + j * DQO_SG, v, sizeof(v));
  }
}
