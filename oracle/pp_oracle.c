/*
 * pp_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain CPU implementation of the steps on either side of DynamiQ's main
 * all-reduce: per-super-group statistics (Section 3.1), their combination over
 * workers (Section 3.1, the "lightweight all-reduce" of Section 3.5), the
 * bit allocation with tied thresholds over W = {2,4,8} or {2,4,8,16} (Section 3.2, Appendix A),
 * the reorder into increasing width order (Section 3.5 "reordering stage"), the
 * means the main stage subtracts (Section 3.1 last paragraph) and the final restore that
 * puts super-groups back and adds the mean back (Section 3.4, last paragraph).
 * Only tests, the smoke check and the benchmark's cpu_baseline leg use it; it
 * shares nothing with the GPU library.
 *
 * Statistics are a plain definition (a mean and a sum of squares), so they are
 * written out in double precision.  Everything that decides an integer (a
 * width, a position) or that is a single rounded fp32 operation is written in
 * exactly the precision both sides agree on; the choices the paper leaves open
 * are stated at each function.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define PPO_SG 256

static float pp_bits_to_f32(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
static uint32_t pp_f32_to_bits(float f) { uint32_t b; memcpy(&b, &f, 4); return b; }

/* fp32 -> bf16, round to nearest, ties to even (finite inputs) */
static uint16_t pp_bf16_rne(float f) {
  uint32_t b = pp_f32_to_bits(f);
  uint32_t keep = b >> 16, rest = b & 0xFFFFu;
  if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
  return (uint16_t)keep;
}
uint16_t ppo_bf16_rne(float f) { return pp_bf16_rne(f); }

static double pp_load(const void *x, int dtype, uint64_t i) {
  if (dtype == 0) return (double)((const float *)x)[i];
  return (double)pp_bits_to_f32((uint32_t)((const uint16_t *)x)[i] << 16);
}

/* Section 3.1: mu_ij = sum(x)/|X_ij|, F_ij = sum(x^2), per super-group of 256 entries.
 * dtype: 0 = fp32, 1 = bf16.  Double precision, left to right. */
void ppo_sg_stats(const void *x, int dtype, uint64_t n_sg, double *mu, double *F) {
  for (uint64_t j = 0; j < n_sg; ++j) {
    double s = 0.0, f = 0.0;
    for (int k = 0; k < PPO_SG; ++k) {
      const double v = pp_load(x, dtype, j * PPO_SG + k);
      s += v;
      f += v * v;
    }
    mu[j] = s / PPO_SG;
    F[j] = f;
  }
}

/* Section 3.1: mu_j = (1/n) sum_i mu_ij, F_j = sum_i F_ij.  Section 3.5: each worker
 * contributes two BF16 numbers per super-group.  Reading: every worker's fp32 statistic
 * is rounded to bf16 (nearest even) before the exchange; the sums run over workers in
 * rank order in fp32; mu_j = sum / n is one fp32 division.  Inputs are row-major [n][J]. */
void ppo_stats_combine(const float *mu_all, const float *F_all, uint32_t n, uint64_t J, float *mu, float *F) {
  for (uint64_t j = 0; j < J; ++j) {
    float sm = 0.0f, sf = 0.0f;
    for (uint32_t i = 0; i < n; ++i) {
      sm = sm + pp_bits_to_f32((uint32_t)pp_bf16_rne(mu_all[(uint64_t)i * J + j]) << 16);
      sf = sf + pp_bits_to_f32((uint32_t)pp_bf16_rne(F_all[(uint64_t)i * J + j]) << 16);
    }
    mu[j] = sm / (float)n;
    F[j] = sf;
  }
}

/* Width of one super-group for a threshold theta = T_{4,8}: Section 3.2 ties the other
 * thresholds to it, T_{2,4} = 17/512 * T_{4,8} and T_{4,8} = 257/2^17 * T_{8,16}; a super-group
 * with F >= T_{b,c} gets at least c bits.  Each tied threshold is one fp32 multiplication of
 * theta by the fp32 constant (17/512 is exact, 2^17/257 is rounded once).  max_width: 8 for
 * W = {2,4,8}, 16 for W = {2,4,8,16}. */
static int pp_width(float F, float theta, int max_width) {
  const float t24 = theta * (17.0f / 512.0f);
  const float t816 = theta * (131072.0f / 257.0f);
  if (max_width == 16 && F >= t816) return 16;
  if (F >= theta) return 8;
  if (F >= t24) return 4;
  return 2;
}
int ppo_width(float F, float theta, int max_width) { return pp_width(F, theta, max_width); }

uint64_t ppo_cost(const float *F, uint64_t J, float theta, int max_width) {
  uint64_t c = 0;
  for (uint64_t j = 0; j < J; ++j) c += (uint64_t)pp_width(F[j], theta, max_width);
  return c;
}

/* Appendix A: one free parameter is searched so that the allocation meets the budget
 * sum_j q_j <= max_code_bits (the per-coordinate code budget times the number of
 * super-groups).  The paper searches the offset u of a logarithmic rule,
 * q = 2^clamp(floor(log2(K log2 F + u))), which is the same family of allocations:
 * z < 4 <=> F < T_{2,4}, z >= 8 <=> F >= (512/17) T_{2,4}.  Reading: instead of u we
 * search T_{4,8} itself over ALL positive fp32 values and +infinity, by bisection on
 * the bit pattern (non-negative floats order like their patterns), and take the
 * smallest threshold whose cost fits: no logarithm, no tolerance, the same answer on
 * any machine.  The cost never increases with the threshold, and +infinity (all at
 * 2 bits) always fits when max_code_bits >= 2J; otherwise -1 is returned.
 * Outputs: widths[j] in {2,4,8(,16)}; returns the threshold's bit pattern. */
int64_t ppo_allocate(const float *F, uint64_t J, uint64_t max_code_bits, int max_width, uint8_t *widths) {
  const uint32_t inf_bits = 0x7F800000u;
  if (ppo_cost(F, J, pp_bits_to_f32(inf_bits), max_width) > max_code_bits) return -1;
  uint32_t lo = 0, hi = inf_bits; /* invariant: cost(hi) fits; lo = 0 stands for "does not fit or not tried" */
  /* smallest pattern in [1, inf_bits] that fits */
  while (hi - lo > 1) {
    const uint32_t mid = lo + (hi - lo) / 2;
    if (ppo_cost(F, J, pp_bits_to_f32(mid), max_width) <= max_code_bits) hi = mid;
    else lo = mid;
  }
  const float theta = pp_bits_to_f32(hi);
  for (uint64_t j = 0; j < J; ++j) widths[j] = (uint8_t)pp_width(F[j], theta, max_width);
  return (int64_t)hi;
}

/* Section 3.5: super-groups are permuted "into a pre-allocated tensor in monotonically
 * increasing bitwidth order".  Reading: stable, i.e. among equal widths the original
 * order is kept.  pos[j] = destination index of super-group j; counts = {n2, n4, n8, n16}. */
static int pp_class(uint8_t w) { return w == 2 ? 0 : w == 4 ? 1 : w == 8 ? 2 : 3; }
void ppo_positions(const uint8_t *widths, uint64_t J, uint32_t *pos, uint32_t counts[4]) {
  uint32_t n[4] = {0, 0, 0, 0};
  for (uint64_t j = 0; j < J; ++j) n[pp_class(widths[j])] += 1;
  uint32_t next[4] = {0, n[0], n[0] + n[1], n[0] + n[1] + n[2]};
  for (uint64_t j = 0; j < J; ++j) pos[j] = next[pp_class(widths[j])]++;
  for (int c = 0; c < 4; ++c) counts[c] = n[c];
}

/* Section 3.5: every worker copies its super-groups into increasing-width order.  A plain
 * permutation of whole super-groups; the bucket has J of them. */
void ppo_reorder(const void *x, int dtype, const uint32_t *pos, uint64_t J, void *out) {
  const size_t esz = dtype == 0 ? 4 : 2;
  for (uint64_t j = 0; j < J; ++j)
    memcpy((uint8_t *)out + (uint64_t)pos[j] * PPO_SG * esz, (const uint8_t *)x + j * PPO_SG * esz, PPO_SG * esz);
}

/* Section 3.1: "each worker normalizes their data by subtracting mu_j from each entry in
 * super-group j".  The main stage does that subtraction itself, in fp32, where an entry
 * enters it, so what it needs is the means in the reordered order.  Reading: a super-group
 * sent uncompressed (16 bits) is not normalized, its mean is taken as zero: a raw bf16 value
 * gains nothing from the subtraction and rounding x - mu back to bf16 would bias the sum.
 * n16 = the number of 16-bit super-groups (they are the last n16 of the reordered bucket). */
void ppo_reorder_mean(const float *mu, const uint32_t *pos, uint64_t J, uint32_t n16, float *mu_main) {
  for (uint64_t j = 0; j < J; ++j) mu_main[pos[j]] = (uint64_t)pos[j] + n16 < J ? mu[j] : 0.0f;
}

/* Section 3.4, last paragraph: "entries are restored to their original order and
 * unnormalized by adding back the mean value".  The main stage returns the SUM over the
 * n workers of the mean-subtracted entries, so what is added back is n times the mean the
 * main stage subtracted (mu_main, in reordered order): one fp32 multiplication per
 * super-group, one fp32 addition per entry.  mu_main NULL: nothing was subtracted, nothing is
 * added (the entries are copied as they are, a zero keeps its sign). */
void ppo_restore(const float *sum, const uint32_t *pos, const float *mu_main, uint32_t n, uint64_t J, float *out) {
  for (uint64_t j = 0; j < J; ++j) {
    const float *src = sum + (uint64_t)pos[j] * PPO_SG;
    if (!mu_main) {
      memcpy(out + j * PPO_SG, src, PPO_SG * sizeof(float));
      continue;
    }
    const float back = (float)n * mu_main[pos[j]];
    for (int k = 0; k < PPO_SG; ++k) out[j * PPO_SG + k] = src[k] + back;
  }
}
