// Host side of libdq: context (level tables, search tables, PRNG key), argument checks and
// the three single-chunk entry points declared in dq.h.
#include <math.h>
#include <string.h>

#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "dq_device.h"

namespace {

thread_local std::string g_hip_error;

bool hip_ok(hipError_t e) {
  if (e == hipSuccess) return true;
  g_hip_error = hipGetErrorString(e);
  return false;
}

// Staging memory of dq_dar_hop_pipelined_static: two halves of a block pipeline.  Every GPU the
// library runs on holds its own copy of this array until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress: the device address of the current GPU's copy
// is resolved once per device (resolve_scratch, called from dq_create) and that pointer is what
// kernels, copies and clears receive.
static __device__ __align__(256) unsigned char scratch[DQ_STATIC_STAGE_BYTES];
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];  // per device ordinal: address of that device's `scratch`, or null
std::mutex g_scratch_mutex;

// The address of `scratch` on `device`, which must be the current device.  nullptr for ordinals this
// table does not cover; *err reports a failed lookup.
void *resolve_scratch(int device, hipError_t *err) {
  *err = hipSuccess;
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void *p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    g_scratch_ptr[device] = p;
  }
  return g_scratch_ptr[device];
}

uint32_t fbits(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  return u;
}

// f(eps, r) = (g^r - 1)/(g^R - 1), g = 1 + 2 eps^2, r = 0..R  (Section 3.3), powers by
// repeated multiplication in double, ends pinned to 0 and 1.
bool build_levels(int R, double g, std::vector<float> &T, std::vector<float> &D) {
  T.assign(R + 1, 0.0f);
  D.assign(R + 1, 0.0f);
  if (R == 1) {
    T[1] = 1.0f;
  } else {
    std::vector<double> pw(R + 1);
    pw[0] = 1.0;
    for (int r = 1; r <= R; ++r) pw[r] = pw[r - 1] * g;
    const double den = pw[R] - 1.0;
    for (int r = 1; r < R; ++r) {
      const double q = (pw[r] - 1.0) / den;
      T[r] = (float)q;
    }
    T[R] = 1.0f;
  }
  for (int r = 0; r < R; ++r) {
    D[r] = T[r + 1] - T[r];
    if (!(D[r] > 0.0f)) return false;
  }
  D[R] = 0.0f;  // at the top level T + u*D = 1 is never below x'
  return true;
}

// Search table over q = round(x * 2^m): the closed bin [(q-1/2)/2^m, (q+1/2)/2^m] holds at
// most one level boundary, so the level at or below x is rc(q) or rc(q)+1.
bool build_search(const std::vector<float> &T, int R, int *m_out, std::vector<uint32_t> &lut) {
  float min_gap = 1.0f;
  for (int r = 0; r < R; ++r) min_gap = fminf(min_gap, T[r + 1] - T[r]);
  for (int m = 1; m <= 12; ++m) {
    const double w = ldexp(1.0, -m);
    if (!(w < (double)min_gap)) continue;
    const int n = (1 << m) + 1;
    lut.assign(2 * (size_t)n, 0u);
    bool ok = true;
    for (int q = 0; q < n && ok; ++q) {
      const double lo = fmax(0.0, ((double)q - 0.5) * w), hi = fmin(1.0, ((double)q + 0.5) * w);
      int rc = 0;
      while (rc < R && (double)T[rc + 1] <= lo) ++rc;
      if (rc > R - 1) ok = false;
      else if (rc + 2 <= R && !((double)T[rc + 2] > hi)) ok = false;
      else {
        lut[2 * q] = fbits(T[rc + 1]);
        lut[2 * q + 1] = (uint32_t)rc;
      }
    }
    if (ok) {
      *m_out = m;
      return true;
    }
  }
  return false;
}

void append_aligned(std::vector<uint32_t> &blob, const std::vector<uint32_t> &part, uint32_t *off) {
  while (blob.size() % 4) blob.push_back(0);
  *off = (uint32_t)blob.size();
  blob.insert(blob.end(), part.begin(), part.end());
}

// The two events of the block pipeline (dq_dar_hop_pipelined*: fork and join of its streams), made
// with the context so that the pipelined calls create nothing.
bool make_events(dq_ctx *ctx) {
  for (int i = 0; i < 2; ++i) ctx->have_event[i] = false;
  for (int i = 0; i < 2; ++i) {
    if (!hip_ok(hipEventCreateWithFlags(&ctx->pipe_event[i], hipEventDisableTiming))) return false;
    ctx->have_event[i] = true;
  }
  ctx->have_events = true;
  return true;
}
void drop_events(dq_ctx *ctx) {
  for (int i = 0; i < 2; ++i) {
    if (ctx->have_event[i]) (void)hipEventDestroy(ctx->pipe_event[i]);
    ctx->have_event[i] = false;
  }
  ctx->have_events = false;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

uint64_t chunk_sgs(const dq_chunk *ch) { return (uint64_t)ch->n_sg[0] + ch->n_sg[1] + ch->n_sg[2] + ch->n_sg[3]; }

dq_status check_chunk(const dq_ctx *ctx, const dq_chunk *ch, uint32_t rank) {
  if (!ctx || !ch) return DQ_EINVAL;
  const uint64_t n = chunk_sgs(ch);
  if (n >= (1ull << 31)) return DQ_EUNSUPPORTED;
  if (rank >= ctx->cfg.n_workers) return DQ_EINVAL;
  if (ch->first_sg + n < ch->first_sg || (ch->first_sg + n) >> 59) return DQ_EINVAL;  // 16*index must fit 64 bits
  return DQ_OK;
}

}  // namespace

dq_status dq::hip_status(hipError_t e) { return hip_ok(e) ? DQ_OK : DQ_EHIP; }

extern "C" {

const char *dq_status_str(dq_status s) {
  switch (s) {
    case DQ_OK: return "ok";
    case DQ_EINVAL: return "invalid argument";
    case DQ_EALIGN: return "pointer not 16-byte aligned";
    case DQ_EUNSUPPORTED: return "unsupported configuration";
    case DQ_EHIP: return "HIP error";
  }
  return "unknown";
}

const char *dq_last_hip_error(void) { return g_hip_error.c_str(); }

dq_status dq_create(const dq_config *cfg, dq_ctx **out) {
  if (!cfg || !out) return DQ_EINVAL;
  *out = nullptr;
  if (cfg->n_workers < 1 || cfg->n_workers > 8192) return DQ_EINVAL;
  if (!(cfg->g4 > 1.0) || !(cfg->g8 > 1.0) || !isfinite(cfg->g4) || !isfinite(cfg->g8)) return DQ_EINVAL;

  const int Rs[3] = {1, 7, 127};
  const double gs[3] = {2.0, cfg->g4, cfg->g8};
  std::vector<uint32_t> blob;
  dq::Params P;
  memset(&P, 0, sizeof(P));
  // Blob layout: the fixed-size tables first, on the constant offsets that dq_device.h declares
  // ([reciprocals][2-bit decode][4-bit decode][4-bit {T,D}][8-bit decode][8-bit {T,D}]), then the
  // two search tables, whose size follows the level sets.
  std::vector<uint32_t> lut[3];
  auto range = [&](int r, uint32_t lo, uint32_t width) {
    P.range_lo[r] = lo;
    P.range_hi[r] = (uint32_t)blob.size();
    P.range_width[r] = width;
  };
  {
    std::vector<uint32_t> rec(256);
    for (int m = 0; m < 128; ++m) {
      const float sig = 1.0f + (float)m / 128.0f;
      const float a = sig / 255.0f, b = 255.0f / sig;
      rec[2 * m] = fbits(a);
      rec[2 * m + 1] = fbits(b);
    }
    uint32_t off;
    append_aligned(blob, rec, &off);
    if (off != dq::kOffRec) return DQ_EINVAL;
    range(0, off, 3);
  }
  const uint32_t want_dec[3] = {dq::kOffDec2, dq::kOffDec4, dq::kOffDec8};
  const uint32_t want_tab[3] = {0, dq::kOffTab4, dq::kOffTab8};
  for (int wi = 0; wi < 3; ++wi) {
    const int R = Rs[wi], b = 2 << wi;  // widths 2, 4, 8
    std::vector<float> T, D;
    if (!build_levels(R, gs[wi], T, D)) return DQ_EINVAL;
    // decode table indexed by one byte of packed codes: the 8/b signed levels it holds,
    // lowest bits first; a code is sign << (b-1) | r
    const int per_byte = 8 / b;
    std::vector<uint32_t> dec((size_t)256 * per_byte);
    for (int byte = 0; byte < 256; ++byte)
      for (int j = 0; j < per_byte; ++j) {
        const int code = (byte >> (j * b)) & ((1 << b) - 1);
        const float t = T[code & R];
        dec[(size_t)byte * per_byte + j] = fbits((code >> (b - 1)) ? -t : t);
      }
    uint32_t off_dec = 0, off_tab = 0;
    append_aligned(blob, dec, &off_dec);
    if (off_dec != want_dec[wi]) return DQ_EINVAL;
    if (wi > 0) {  // levels {0,1} need no search
      std::vector<uint32_t> tab(2 * (size_t)(R + 1));
      for (int r = 0; r <= R; ++r) {
        tab[2 * r] = fbits(T[r]);
        tab[2 * r + 1] = fbits(D[r]);
      }
      // at the top level nothing rounds up: T + u*D is held above every x' the kernels can form (they
      // do not clamp x' to 1; it can exceed 1 by an ulp when the reciprocal of the group maximum is denormal)
      tab[2 * R] = fbits(2.0f);
      append_aligned(blob, tab, &off_tab);
      if (off_tab != want_tab[wi]) return DQ_EINVAL;
      int m = 0;
      if (!build_search(T, R, &m, lut[wi])) return DQ_EUNSUPPORTED;
      P.magic[wi] = (float)ldexp(1.0, 23 - m);
    }
    while (blob.size() % 4) blob.push_back(0);
    range(1 + wi, off_dec, (uint32_t)wi);
  }
  {
    uint32_t off;
    append_aligned(blob, lut[1], &off);
    if (off != dq::kOffLut4) return DQ_EINVAL;
    while (blob.size() % 4) blob.push_back(0);
    range(4, off, 1);
    append_aligned(blob, lut[2], &P.off_lut8);
    while (blob.size() % 4) blob.push_back(0);
    range(5, P.off_lut8, 2);
  }
  if (blob.size() * 4 > 60 * 1024) return DQ_EUNSUPPORTED;

  dq_ctx *ctx = new (std::nothrow) dq_ctx;
  if (!ctx) return DQ_EINVAL;
  ctx->cfg = *cfg;
  ctx->blob_dev = nullptr;
  ctx->have_events = false;
  for (int i = 0; i < 2; ++i) ctx->have_event[i] = false;
  ctx->static_stage = nullptr;
  hipDeviceProp_t prop;
  hipError_t sym_err = hipSuccess;
  if (!hip_ok(hipGetDevice(&ctx->device)) || !hip_ok(hipGetDeviceProperties(&prop, ctx->device)) ||
      !hip_ok(hipMalloc(&ctx->blob_dev, blob.size() * 4)) ||
      !hip_ok(hipMemcpy(ctx->blob_dev, blob.data(), blob.size() * 4, hipMemcpyHostToDevice)) ||
      ((ctx->static_stage = resolve_scratch(ctx->device, &sym_err)), !hip_ok(sym_err)) || !make_events(ctx)) {
    if (ctx->blob_dev) (void)hipFree(ctx->blob_dev);
    drop_events(ctx);
    delete ctx;
    return DQ_EHIP;
  }
  {  // the kernels address their tables from LDS byte 0: true as long as they have no static LDS
    size_t static_lds = 0;
    if (!hip_ok(dq::static_lds_bytes(&static_lds)) || static_lds != 0) {
      if (static_lds != 0) g_hip_error = "codec kernels were built with static LDS: table addresses would be off";
      (void)hipFree(ctx->blob_dev);
      drop_events(ctx);
      delete ctx;
      return DQ_EHIP;
    }
  }
  ctx->n_cu = (uint32_t)prop.multiProcessorCount;
  // five blocks of four waves per CU: measured against 4, 6 and 7 (fewer waves hide too little of each other's
  // waits, more of them contend at the start of a short launch and pay the per-wave set-up more often)
  uint32_t per_cu = 5;
  const char *env = getenv("DQ_BLOCKS_PER_CU");  // tuning / test knob, read once per context
  if (env && atoi(env) >= 1 && atoi(env) <= 64) per_cu = (uint32_t)atoi(env);
  ctx->grid_blocks = ctx->n_cu * per_cu;
  P.blob = ctx->blob_dev;
  P.blob_dwords = (uint32_t)blob.size();
  P.key0 = (uint32_t)cfg->seed;
  P.key1 = (uint32_t)(cfg->seed >> 32);
  P.round = cfg->round;
  P.n_workers = cfg->n_workers;
  P.n_mask = (cfg->n_workers & (cfg->n_workers - 1)) == 0 ? cfg->n_workers - 1 : 0xFFFFFFFFu;
  while ((1u << P.perm_bits) < cfg->n_workers) ++P.perm_bits;  // the shared permutation mixes integers of this many bits
  P.inv_n = 1.0f / (float)cfg->n_workers;
  if (cfg->independent_rounding) {  // the case n = 1 of the same arithmetic: one interval, slot 0
    P.inv_n = 1.0f;
    P.n_mask = 0;
  }
  P.s_n = P.inv_n * (1.0f / 256.0f);
  ctx->params = P;
  *out = ctx;
  return DQ_OK;
}

void dq_destroy(dq_ctx *ctx) {
  if (!ctx) return;
  if (ctx->blob_dev) (void)hipFree(ctx->blob_dev);
  drop_events(ctx);
  delete ctx;
}

dq_status dq_stream_probe(dq_ctx *ctx, const void *in, size_t in_bytes, void *out, size_t out_bytes, void *hip_stream) {
  if (!ctx || !in || !out || in_bytes == 0 || out_bytes == 0 || out_bytes > in_bytes) return DQ_EINVAL;
  if ((in_bytes | out_bytes) & 15u) return DQ_EINVAL;
  if (!aligned16(in) || !aligned16(out)) return DQ_EALIGN;
  return dq::hip_status(dq::stream_probe(in, in_bytes, out, out_bytes, ctx->n_cu, (hipStream_t)hip_stream));
}

dq_status dq_set_round(dq_ctx *ctx, uint32_t round) {
  if (!ctx) return DQ_EINVAL;
  ctx->cfg.round = round;
  ctx->params.round = round;
  return DQ_OK;
}

size_t dq_packed_bytes(const dq_chunk *ch) {
  if (!ch) return 0;
  const size_t n = (size_t)ch->n_sg[0] + ch->n_sg[1] + ch->n_sg[2];  // coded super-groups carry scales
  const size_t sz = 64 * (size_t)ch->n_sg[0] + 128 * (size_t)ch->n_sg[1] + 256 * (size_t)ch->n_sg[2] +
                    512 * (size_t)ch->n_sg[3] + 18 * n;
  return (sz + 15) & ~(size_t)15;
}

// Checks a local operand and fills the job's local fields from it.
static dq_status take_local(const dq_local *l, dq::Job *j) {
  if (!l->data || (l->dtype != DQ_F32 && l->dtype != DQ_BF16)) return DQ_EINVAL;
  if (!aligned16(l->data) || !aligned4(l->mu) || !aligned4(l->sg_index)) return DQ_EALIGN;
  j->local = l->data;
  j->mu = l->mu;
  j->src = l->sg_index;
  return DQ_OK;
}

dq_status dq_compress(dq_ctx *ctx, const dq_local *local, const dq_chunk *chunk, uint32_t rank, void *packed_out,
                      void *hip_stream) {
  dq_status st = check_chunk(ctx, chunk, rank);
  if (st != DQ_OK) return st;
  if (chunk_sgs(chunk) == 0) return DQ_OK;  // nothing to do
  if (!local || !packed_out) return DQ_EINVAL;
  if (!aligned16(packed_out)) return DQ_EALIGN;
  dq::Job j = dq::make_job(nullptr, nullptr, nullptr, packed_out, chunk->first_sg, chunk->n_sg, rank);
  if ((st = take_local(local, &j)) != DQ_OK) return st;
  return dq::hip_status(dq::launch_one(dq::kCompress, local->dtype, true, j, ctx->params, ctx->grid_blocks, (hipStream_t)hip_stream));
}

dq_status dq_dar_hop(dq_ctx *ctx, const void *packed_in, const dq_local *local, const dq_chunk *chunk, uint32_t rank,
                     void *packed_out, void *hip_stream) {
  dq_status st = check_chunk(ctx, chunk, rank);
  if (st != DQ_OK) return st;
  if (chunk_sgs(chunk) == 0) return DQ_OK;
  if (!packed_in || !local || !packed_out) return DQ_EINVAL;
  if (!aligned16(packed_in) || !aligned16(packed_out)) return DQ_EALIGN;
  dq::Job j = dq::make_job((const uint8_t *)packed_in, nullptr, nullptr, packed_out, chunk->first_sg, chunk->n_sg, rank);
  if ((st = take_local(local, &j)) != DQ_OK) return st;
  return dq::hip_status(dq::launch_one(dq::kDar, local->dtype, true, j, ctx->params, ctx->grid_blocks, (hipStream_t)hip_stream));
}

dq_status dq_decompress(dq_ctx *ctx, const void *packed_in, const dq_local *local_or_null, const dq_chunk *chunk,
                        float *out, void *hip_stream) {
  dq_status st = check_chunk(ctx, chunk, 0);
  if (st != DQ_OK) return st;
  if (chunk_sgs(chunk) == 0) return DQ_OK;
  if (!packed_in || !out) return DQ_EINVAL;
  if (!aligned16(packed_in) || !aligned16(out)) return DQ_EALIGN;
  dq::Job j = dq::make_job((const uint8_t *)packed_in, nullptr, nullptr, out, chunk->first_sg, chunk->n_sg, 0);
  if (local_or_null && (st = take_local(local_or_null, &j)) != DQ_OK) return st;
  // a gathered local cannot be accumulated in place: other super-groups' inputs would be overwritten
  if (local_or_null && local_or_null->sg_index && local_or_null->data == (const void *)out) return DQ_EINVAL;
  return dq::hip_status(dq::launch_one(dq::kDecompress, local_or_null ? local_or_null->dtype : DQ_F32, local_or_null != nullptr,
                                       j, ctx->params, ctx->grid_blocks, (hipStream_t)hip_stream));
}

dq_status dq_decompress_restore(dq_ctx *ctx, const void *packed_in, const dq_local *local_or_null, const dq_chunk *chunk,
                                const uint32_t *origin, const float *mu_back_or_null, float *out_base, void *hip_stream) {
  dq_status st = check_chunk(ctx, chunk, 0);
  if (st != DQ_OK) return st;
  if (chunk_sgs(chunk) == 0) return DQ_OK;
  if (!packed_in || !out_base || !origin) return DQ_EINVAL;
  if (!aligned16(packed_in) || !aligned16(out_base) || !aligned4(origin) || !aligned4(mu_back_or_null)) return DQ_EALIGN;
  dq::Job j = dq::make_job((const uint8_t *)packed_in, nullptr, nullptr, out_base, chunk->first_sg, chunk->n_sg, 0);
  if (local_or_null && (st = take_local(local_or_null, &j)) != DQ_OK) return st;
  if (local_or_null && local_or_null->data == (const void *)out_base) return DQ_EINVAL;  // scattered stores: not in place
  j.dest = origin;
  j.back = mu_back_or_null;
  return dq::hip_status(dq::launch_one(dq::kDecompress, local_or_null ? local_or_null->dtype : DQ_F32, local_or_null != nullptr,
                                       j, ctx->params, ctx->grid_blocks, (hipStream_t)hip_stream));
}

}  // extern "C"

// ---- block-wise pipelining -------------------------------------------------------------

namespace {

// Block b of a chunk cut every block_sg super-groups: a chunk of its own.
dq_chunk block_of(const dq_chunk *ch, uint32_t block_sg, uint64_t b) {
  uint64_t edges[5] = {0, 0, 0, 0, 0};
  for (int w = 0; w < 4; ++w) edges[w + 1] = edges[w] + ch->n_sg[w];
  const uint64_t lo = b * block_sg, hi = lo + block_sg < edges[4] ? lo + block_sg : edges[4];
  dq_chunk out;
  out.first_sg = ch->first_sg + lo;
  for (int w = 0; w < 4; ++w) {
    const uint64_t a = lo > edges[w] ? lo : edges[w], e = hi < edges[w + 1] ? hi : edges[w + 1];
    out.n_sg[w] = e > a ? (uint32_t)(e - a) : 0;
  }
  return out;
}

size_t wire_slot(const dq_chunk *blk) { return (dq_packed_bytes(blk) + 255) & ~(size_t)255; }

}  // namespace

extern "C" {

size_t dq_pipelined_wire_bytes(const dq_chunk *chunk, uint32_t block_sg) {
  if (!chunk || block_sg == 0) return 0;
  const uint64_t n = chunk_sgs(chunk), blocks = (n + block_sg - 1) / block_sg;
  size_t total = 0;
  for (uint64_t b = 0; b < blocks; ++b) {
    const dq_chunk blk = block_of(chunk, block_sg, b);
    total += wire_slot(&blk);
  }
  return total;
}

size_t dq_pipelined_stage_bytes(const dq_chunk *chunk, uint32_t block_sg) {
  if (!chunk || block_sg == 0) return 0;
  const uint64_t n = chunk_sgs(chunk), blocks = (n + block_sg - 1) / block_sg;
  size_t biggest = 0;
  for (uint64_t b = 0; b < blocks; ++b) {
    const dq_chunk blk = block_of(chunk, block_sg, b);
    const size_t s = wire_slot(&blk);
    if (s > biggest) biggest = s;
  }
  return 2 * biggest;
}

static dq_status pipelined_hop(dq_ctx *ctx, const void *wire_in, const dq_local *local, const dq_chunk *chunk,
                               uint32_t rank, uint32_t block_sg, void *stage, void *wire_out, void *compute_stream,
                               void *copy_stream);

dq_status dq_dar_hop_pipelined(dq_ctx *ctx, const void *wire_in, const dq_local *local, const dq_chunk *chunk,
                               uint32_t rank, uint32_t block_sg, void *stage, void *wire_out, void *compute_stream,
                               void *copy_stream) {
  return pipelined_hop(ctx, wire_in, local, chunk, rank, block_sg, stage, wire_out, compute_stream, copy_stream);
}

dq_status dq_dar_hop_pipelined_static(dq_ctx *ctx, const void *wire_in, const dq_local *local, const dq_chunk *chunk,
                                      uint32_t rank, uint32_t block_sg, void *wire_out, void *compute_stream,
                                      void *copy_stream) {
  if (!ctx || !chunk || block_sg == 0) return DQ_EINVAL;
  const size_t need = dq_pipelined_stage_bytes(chunk, block_sg);
  if (need > (size_t)DQ_STATIC_STAGE_BYTES) {
    g_hip_error = "dq_dar_hop_pipelined_static: two blocks of " + std::to_string(block_sg) + " super-groups need " +
                  std::to_string(need) + " bytes of staging, the static scratch holds " +
                  std::to_string((size_t)DQ_STATIC_STAGE_BYTES) + ": use smaller blocks or dq_dar_hop_pipelined";
    return DQ_EUNSUPPORTED;
  }
  int device = -1;
  if (!hip_ok(hipGetDevice(&device))) return DQ_EHIP;
  if (device != ctx->device) {  // the scratch pointer kept in the context belongs to the context's GPU
    g_hip_error = "dq_dar_hop_pipelined_static: the context was made on another device than the current one";
    return DQ_EINVAL;
  }
  if (!ctx->static_stage || !ctx->have_events) {
    g_hip_error = "dq_dar_hop_pipelined_static: no static scratch on this device ordinal";
    return DQ_EUNSUPPORTED;
  }
  return pipelined_hop(ctx, wire_in, local, chunk, rank, block_sg, ctx->static_stage, wire_out, compute_stream, copy_stream);
}

static dq_status pipelined_hop(dq_ctx *ctx, const void *wire_in, const dq_local *local, const dq_chunk *chunk,
                               uint32_t rank, uint32_t block_sg, void *stage, void *wire_out, void *compute_stream,
                               void *copy_stream) {
  dq_status st = check_chunk(ctx, chunk, rank);
  if (st != DQ_OK) return st;
  const uint64_t n = chunk_sgs(chunk);
  if (n == 0) return DQ_OK;
  if (!local || !stage || !wire_out || block_sg == 0) return DQ_EINVAL;
  if (compute_stream == copy_stream) return DQ_EINVAL;  // the overlap needs two streams
  if (!aligned16(wire_in) || !aligned16(stage) || !aligned16(wire_out)) return DQ_EALIGN;
  dq::Job whole = dq::make_job(nullptr, nullptr, nullptr, nullptr, chunk->first_sg, chunk->n_sg, rank);
  if ((st = take_local(local, &whole)) != DQ_OK) return st;
  const dq_dtype dtype = local->dtype;
  hipStream_t lane[2] = {(hipStream_t)compute_stream, (hipStream_t)copy_stream};
  if (!ctx->have_events) return DQ_EHIP;  // made in dq_create
  const size_t half = dq_pipelined_stage_bytes(chunk, block_sg) / 2;
  const size_t es = dtype == DQ_F32 ? 4 : 2;
  const uint64_t blocks = (n + block_sg - 1) / block_sg;
  // Block b is encoded into half b mod 2 of the stage and then sent, both on stream b mod 2: the order
  // inside a stream keeps a half from being overwritten before it has left, the two streams overlap
  // the encoding of one block with the transfer of the one before, and no event is needed per block
  // (seven runtime calls per block took 26 us of host time, four times what a block's kernel takes).
  // The second stream starts after what the first has queued so far (the inputs) ...
  if (blocks > 1 && (!hip_ok(hipEventRecord(ctx->pipe_event[0], lane[0])) ||
                     !hip_ok(hipStreamWaitEvent(lane[1], ctx->pipe_event[0], 0))))
    return DQ_EHIP;
  size_t wire_off = 0;
  for (uint64_t b = 0; b < blocks; ++b) {
    const dq_chunk blk = block_of(chunk, block_sg, b);
    const size_t bytes = dq_packed_bytes(&blk);
    const size_t coded = (size_t)blk.n_sg[0] + blk.n_sg[1] + blk.n_sg[2];
    const size_t valid = 64 * (size_t)blk.n_sg[0] + 128 * (size_t)blk.n_sg[1] + 256 * (size_t)blk.n_sg[2] +
                         512 * (size_t)blk.n_sg[3] + 18 * coded;  // the rest of `bytes` is padding
    const int slot = (int)(b & 1);
    uint8_t *stg = static_cast<uint8_t *>(stage) + slot * half;
    // block b of the chunk: its slice of a contiguous local, or its slice of the indices into a gathered one
    const uint64_t sg_first = b * (uint64_t)block_sg;
    dq::Job j = dq::make_job(wire_in ? static_cast<const uint8_t *>(wire_in) + wire_off : nullptr,
                             whole.src ? whole.local : static_cast<const uint8_t *>(whole.local) + sg_first * 256 * es,
                             whole.mu ? whole.mu + sg_first : nullptr, stg, blk.first_sg, blk.n_sg, rank);
    j.src = whole.src ? whole.src + sg_first : nullptr;
    if (!hip_ok(dq::launch_one(wire_in ? dq::kDar : dq::kCompress, dtype, true, j, ctx->params, ctx->grid_blocks, lane[slot])))
      return DQ_EHIP;
    // the transfer: a device copy standing in for the wire; it writes the block's padding as zero, which
    // the codec kernels leave untouched in the stage
    if (!hip_ok(dq::wire_copy(static_cast<uint8_t *>(wire_out) + wire_off, stg, bytes, valid, lane[slot]))) return DQ_EHIP;
    wire_off += wire_slot(&blk);
  }
  // ... and whoever waits for the first stream also waits for the second
  if (blocks > 1 && (!hip_ok(hipEventRecord(ctx->pipe_event[1], lane[1])) ||
                     !hip_ok(hipStreamWaitEvent(lane[0], ctx->pipe_event[1], 0))))
    return DQ_EHIP;
  return DQ_OK;
}

}  // extern "C"
